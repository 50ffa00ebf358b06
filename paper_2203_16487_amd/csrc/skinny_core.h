// Building blocks of the small-batch (at most 32 rows) decoder kernels: LDS carve-up, the
// hidden-state prologue, K-split weight-streaming products on MFMA 16x16x32 and their
// reduction.  Used by the per-projection kernels and by the single resident kernel.
#pragma once
#include <type_traits>
#include "attn_core.h"

namespace sd {

constexpr int kSkThreads = 256;
constexpr int kSkRows = 32;          // activation rows a block can hold (2 MFMA column tiles)
constexpr int kSkAttnWaves = 8;      // waves of the attention + O kernel (one (sequence, head) pair each)
constexpr int kSkPad = 8;            // bf16 padding of an activation row in LDS (bank spread)

// LDS carve-up (dynamic): hb bf16 [32][d + 8] | hown f32 [2][32][16] | red f32 [4][16][33] | Vs
template <int PER>
struct SkLds {
  static constexpr int d = 64 * PER;
  static constexpr int kPitch = d + kSkPad;
  static constexpr size_t kHb = (size_t)kSkRows * kPitch * 2;
  static constexpr size_t kOwn = (size_t)2 * kSkRows * 16 * 4;
  static constexpr size_t kRed = (size_t)4 * 16 * 33 * 4;
  static constexpr size_t kVs = (size_t)kSkAttnWaves * 32 * kVtPitch * 2;
  static constexpr size_t kBytes = kHb + kOwn + kRed + kVs;
  static constexpr size_t kBytesNoAttn = kHb + kOwn + kRed;   // kernels without attention: Vs (last) left out
  bf16* hb; float* hown; float* red; bf16 (*vs)[32][kVtPitch];
  __device__ explicit SkLds(char* base) {
    hb = reinterpret_cast<bf16*>(base);
    hown = reinterpret_cast<float*>(base + kHb);
    red = reinterpret_cast<float*>(base + kHb + kOwn);
    vs = reinterpret_cast<bf16 (*)[32][kVtPitch]>(base + kHb + kOwn + kRed);
  }
};

// Hidden state of the R rows = what `src` describes; bf16 copy of all columns -> hb, fp32 copy
// of columns [n0, n0 + 16) -> hown (for residual adds).  Rows R .. nrows-1 of hb / hown are not
// written: in the products that follow an activation row only feeds its own output row, and
// every consumer drops output rows >= R.
// A wave takes rows base, base + STRIDE, ...; it requests the data of RU of them (and the
// LayerNorm parameters, once) before it reduces any, so the prologue costs one memory round
// trip for RU rows per wave.
// COH: the fp32 rows were written by other workgroups of the running kernel.  n0b: a second
// 16-column residual slice (slot 1 of hown, [2][32][16]); negative: none.
// A lane holds VEC consecutive columns per 64*VEC-column group (VEC = 4 when d % 256 == 0), so a
// row is fetched with 16-byte loads: the prologue's cost is the number of load instructions
// the CU has to issue, not their bytes.
template <int PER, bool COH = false, int RU = 4, int STRIDE = 4>
struct SkHidden {
  static constexpr int d = 64 * PER, pitch = d + kSkPad;
  static constexpr int VEC = PER % 4 == 0 ? 4 : (PER % 2 == 0 ? 2 : 1);
  static constexpr int NV = PER / VEC;                      // vector loads per row and lane
  // LayerNorm parameters exactly as loaded (whole 2*VEC-byte words): taking them apart where
  // they are requested would make the kernel wait for them there
  template <int N> struct RawT { typedef unsigned short type; };
  template <> struct RawT<2> { typedef unsigned type; };
  template <> struct RawT<4> { typedef unsigned long long type; };
  typedef typename RawT<VEC>::type RawV;
  RawV gg[NV], bb[NV];
  float v[RU][PER];
  __device__ __forceinline__ static float raw_at(const RawV (&p)[NV], int i) {
    return __builtin_bit_cast(float, (unsigned)((p[i / VEC] >> (16 * (i % VEC))) & 0xffffu) << 16);   // bf16 -> fp32
  }
  // column of element i of this lane
  __device__ __forceinline__ static int col(int i, int lane) { return (i / VEC) * (64 * VEC) + lane * VEC + i % VEC; }

  template <class T>
  __device__ __forceinline__ static void load_vec(const T* p, float* out) {   // VEC values -> fp32
    if constexpr (sizeof(T) == 4) {
      if constexpr (VEC == 4) {
        f32x4 t;
        if (COH) {
          const unsigned long long* q = reinterpret_cast<const unsigned long long*>(p);
          unsigned long long u[2] = {__hip_atomic_load(q, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT),
                                     __hip_atomic_load(q + 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT)};
          __builtin_memcpy(&t, u, 16);
        } else {
          t = *reinterpret_cast<const f32x4*>(p);
        }
        out[0] = t[0]; out[1] = t[1]; out[2] = t[2]; out[3] = t[3];
      } else if constexpr (VEC == 2) {
        float t[2];
        if (COH) {
          unsigned long long u = __hip_atomic_load(reinterpret_cast<const unsigned long long*>(p), __ATOMIC_RELAXED,
                                                   __HIP_MEMORY_SCOPE_AGENT);
          __builtin_memcpy(t, &u, 8);
        } else {
          __builtin_memcpy(t, p, 8);
        }
        out[0] = t[0]; out[1] = t[1];
      } else {
        out[0] = COH ? ld_coh(p) : p[0];
      }
    } else {   // bf16 (read-only data: never written by the running kernel)
      if constexpr (VEC == 4) {
        const bf16x4 t = *reinterpret_cast<const bf16x4*>(p);
        out[0] = (float)t[0]; out[1] = (float)t[1]; out[2] = (float)t[2]; out[3] = (float)t[3];
      } else if constexpr (VEC == 2) {
        const bf16x2 t = *reinterpret_cast<const bf16x2*>(p);
        out[0] = (float)t[0]; out[1] = (float)t[1];
      } else {
        out[0] = (float)p[0];
      }
    }
  }

  // LayerNorm parameters of this lane's columns (once per kernel): requested, not waited for
  __device__ __forceinline__ void params(const SkSrc& s) {
    const int lane = threadIdx.x & 63;
    if (s.mode == 2) {
#pragma unroll
      for (int j = 0; j < NV; ++j) {
        gg[j] = *reinterpret_cast<const RawV*>(s.g + col(j * VEC, lane));
        bb[j] = *reinterpret_cast<const RawV*>(s.b + col(j * VEC, lane));
      }
    }
  }
  // request rows base, base + STRIDE, ... (RU rows, clamped to R - 1): nothing is waited for
  __device__ __forceinline__ void load(const SkSrc& s, int R, int base) {
    const int lane = threadIdx.x & 63;
    if (s.mode == 0) {
      int tok[RU], pos[RU];
#pragma unroll
      for (int u = 0; u < RU; ++u) {
        const int r = min(base + STRIDE * u, R - 1);
        tok[u] = s.tok[r]; pos[u] = s.pos[r];
      }
      const float sc = sqrtf((float)d);
#pragma unroll
      for (int u = 0; u < RU; ++u) {
        const bf16* e = s.E + (size_t)tok[u] * d;
        const float* p = s.pe + (size_t)pos[u] * d;
#pragma unroll
        for (int j = 0; j < NV; ++j) {
          float ev[VEC], pv[VEC];
          load_vec(e + col(j * VEC, lane), ev);
          SkHidden<PER, false, RU, STRIDE>::load_vec(p + col(j * VEC, lane), pv);
#pragma unroll
          for (int i = 0; i < VEC; ++i) v[u][j * VEC + i] = ev[i] * sc + pv[i];
        }
      }
    } else {
#pragma unroll
      for (int u = 0; u < RU; ++u) {
        const int r = base + STRIDE * u;
        if (r < R) {   // (same for the whole wave)
#pragma unroll
          for (int j = 0; j < NV; ++j) load_vec(s.xs + (size_t)r * d + col(j * VEC, lane), v[u] + j * VEC);
        }
      }
    }
  }
  // normalise the requested rows and write them out (rows >= R: nothing, see above)
  __device__ __forceinline__ void finish(const SkSrc& s, int R, int nrows, int base, bf16* hb, float* hown, int n0,
                                         bool want_hb, int n0b) {
    normalize(s, R, nrows, base);
    write(R, nrows, base, hb, hown, n0, want_hb, n0b);
  }
  __device__ __forceinline__ void normalize(const SkSrc& s, int R, int nrows, int base) {
    const int rmax = min(R, nrows);
    if (s.mode == 2) {
      if (base + STRIDE * 2 < rmax) {
        // more than two rows of this wave are in use: all RU are reduced (the unused ones on
        // whatever their registers hold; they are not written), one kind of reduction after the
        // other, so that the independent reductions overlap
        float mean[RU], rstd[RU];
#pragma unroll
        for (int u = 0; u < RU; ++u) {
          float sum = 0.f;
#pragma unroll
          for (int i = 0; i < PER; ++i) sum += v[u][i];
          mean[u] = wave_sum(sum) / (float)d;
        }
#pragma unroll
        for (int u = 0; u < RU; ++u) {
          float q = 0.f;
#pragma unroll
          for (int i = 0; i < PER; ++i) { float t = v[u][i] - mean[u]; q += t * t; }
          rstd[u] = fast_rsqrt(wave_sum(q) / (float)d + 1e-5f);
        }
#pragma unroll
        for (int u = 0; u < RU; ++u)
#pragma unroll
          for (int i = 0; i < PER; ++i) v[u][i] = (v[u][i] - mean[u]) * rstd[u] * raw_at(gg, i) + raw_at(bb, i);
      } else {
#pragma unroll
        for (int u = 0; u < RU; ++u) {
          if (base + STRIDE * u >= rmax) continue;   // (same for the whole wave)
          float sum = 0.f;
#pragma unroll
          for (int i = 0; i < PER; ++i) sum += v[u][i];
          const float mean = wave_sum(sum) / (float)d;
          float q = 0.f;
#pragma unroll
          for (int i = 0; i < PER; ++i) { float t = v[u][i] - mean; q += t * t; }
          const float rstd = fast_rsqrt(wave_sum(q) / (float)d + 1e-5f);
#pragma unroll
          for (int i = 0; i < PER; ++i) v[u][i] = (v[u][i] - mean) * rstd * raw_at(gg, i) + raw_at(bb, i);
        }
      }
    }
  }
  __device__ __forceinline__ void write(int R, int nrows, int base, bf16* hb, float* hown, int n0, bool want_hb,
                                        int n0b) {
    const int lane = threadIdx.x & 63;
    const int rmax = min(R, nrows);
#pragma unroll
    for (int u = 0; u < RU; ++u) {
      const int r = base + STRIDE * u;
      if (r >= rmax) continue;
#pragma unroll
      for (int j = 0; j < NV; ++j) {
        const int c0 = col(j * VEC, lane);
        if (want_hb) {
          bf16 packed[VEC];
#pragma unroll
          for (int i = 0; i < VEC; ++i) packed[i] = (bf16)v[u][j * VEC + i];
          __builtin_memcpy(hb + r * pitch + c0, packed, 2 * VEC);   // 2*VEC-byte aligned: pitch, c0 multiples of VEC
        }
        // the 16-column slices start at multiples of 16, so a lane's VEC columns are in or out together
        if (c0 >= n0 && c0 < n0 + 16) {
#pragma unroll
          for (int i = 0; i < VEC; ++i) hown[r * 16 + c0 - n0 + i] = v[u][j * VEC + i];
        }
        if (c0 >= n0b && c0 < n0b + 16) {
#pragma unroll
          for (int i = 0; i < VEC; ++i) hown[kSkRows * 16 + r * 16 + c0 - n0b + i] = v[u][j * VEC + i];
        }
      }
    }
  }
};

// Hidden state with a pending sub-layer sum: the sub-layer before this kernel was computed in
// slices (one per head, or per slice of the FFN width), each slice leaving a partial result
// part[p] [R][d] (fp32).  What the kernel needs is
//     y = base + pbias + part[0] + part[1] + ... + part[np-1]      (summed in this order, always)
//     hidden = LayerNorm_{g2,b2}(y)
// with base = the hidden state that SkSrc's first fields describe (the sub-layer's input: the
// residual).  Every block recomputes it; block 0 also stores y to xs_out (the `xs` of the next
// kernel's base).  A wave takes rows wave, wave + NW, ..., one at a time: the row's base data and
// all its partial slices are requested before the first reduction.
template <int PER, int NW, int PREG = 128>
__device__ __forceinline__ void sk_hidden_sum(const SkSrc& s, int R, int nrows, bf16* hb, float* hown, int n0,
                                              bool want_hb, int n0b) {
  typedef SkHidden<PER, false, 1, NW> HS;
  constexpr int d = 64 * PER, VEC = HS::VEC, NV = HS::NV;
  constexpr int PB = (PREG / PER) < 1 ? 1 : (PREG / PER);   // partial slices held in registers at a time
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  if (wave >= NW) return;
  HS hs;
  hs.params(s);
  float g2[PER], b2[PER], pb[PER];
#pragma unroll
  for (int j = 0; j < NV; ++j) {
    HS::load_vec(s.g2 + HS::col(j * VEC, lane), g2 + j * VEC);
    HS::load_vec(s.b2 + HS::col(j * VEC, lane), b2 + j * VEC);
    HS::load_vec(s.pbias + HS::col(j * VEC, lane), pb + j * VEC);
  }
  const int rmax = min(R, nrows);
  for (int r = wave; r < rmax; r += NW) {
    hs.load(s, R, r);
    float acc[PER];
    bool first = true;
    for (int p0 = 0; p0 < s.np; p0 += PB) {
      float pv[PB][PER];
#pragma unroll
      for (int u = 0; u < PB; ++u) {
        const int p = min(p0 + u, s.np - 1);
        const float* src = s.part + (size_t)p * s.part_stride + (size_t)r * d;
#pragma unroll
        for (int j = 0; j < NV; ++j) HS::load_vec(src + HS::col(j * VEC, lane), pv[u] + j * VEC);
      }
      if (first) {
        hs.normalize(s, R, nrows, r);
#pragma unroll
        for (int i = 0; i < PER; ++i) acc[i] = hs.v[0][i] + pb[i];
        first = false;
      }
#pragma unroll
      for (int u = 0; u < PB; ++u)
        if (p0 + u < s.np) {
#pragma unroll
          for (int i = 0; i < PER; ++i) acc[i] += pv[u][i];
        }
    }
    if (blockIdx.x == 0 && s.xs_out) {
#pragma unroll
      for (int j = 0; j < NV; ++j) {
        float* dst = s.xs_out + (size_t)r * d + HS::col(j * VEC, lane);
#pragma unroll
        for (int i = 0; i < VEC; ++i) dst[i] = acc[j * VEC + i];
      }
    }
    float sum = 0.f;
#pragma unroll
    for (int i = 0; i < PER; ++i) sum += acc[i];
    const float mean = wave_sum(sum) / (float)d;
    float q = 0.f;
#pragma unroll
    for (int i = 0; i < PER; ++i) { const float t = acc[i] - mean; q += t * t; }
    const float rstd = fast_rsqrt(wave_sum(q) / (float)d + 1e-5f);
#pragma unroll
    for (int i = 0; i < PER; ++i) hs.v[0][i] = (acc[i] - mean) * rstd * g2[i] + b2[i];
    hs.write(R, nrows, r, hb, hown, n0, want_hb, n0b);
  }
}

template <int PER, bool COH = false>
__device__ __forceinline__ void sk_hidden(const SkSrc& s, int R, int nrows, bf16* hb, float* hown, int n0,
                                          bool want_hb, int n0b = -64) {
  if (!COH && s.np > 0) {   // (same for the whole grid)
    sk_hidden_sum<PER, 4>(s, R, nrows, hb, hown, n0, want_hb, n0b);
    return;
  }
  const int wave = (threadIdx.x >> 6) & 3;
  if (PER <= 8 && nrows > 16) {   // eight rows per wave at once: still one round trip for 32 rows
    SkHidden<PER, COH, 8> hs;
    hs.params(s);
    hs.load(s, R, wave);
    hs.finish(s, R, nrows, wave, hb, hown, n0, want_hb, n0b);
    return;
  }
  SkHidden<PER, COH> hs;
  hs.params(s);
  for (int base = wave; base < nrows; base += 16) {
    hs.load(s, R, base);
    hs.finish(s, R, nrows, base, hb, hown, n0, want_hb, n0b);
  }
}

// Weight operands of this wave: rows n0 + lane%16 of W, k range [k0, k0 + 32*S).  sk_wload only
// issues the loads -- kernels call it first thing, so the weights travel while the prologue
// (LayerNorm, attention) runs; sk_mma consumes them:
//   acc[t] += W[n0 + i][k] . B_t[j][k],  getB(t, k) = 8 bf16 of activation row t*16 + lane%16 at k.
// Step counts and the second row tile are compile-time, so the MFMA sequence is straight-line.
// four consecutive bf16 (8-byte aligned) stored so that other waves' coherent loads see them
__device__ __forceinline__ void st_coh4(bf16* p, const float (&v)[4]) {
  bf16x4 t;
#pragma unroll
  for (int i = 0; i < 4; ++i) t[i] = (bf16)v[i];
  unsigned long long u;
  __builtin_memcpy(&u, &t, 8);
  __hip_atomic_store(reinterpret_cast<unsigned long long*>(p), u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

constexpr int kSkW = 16;   // most steps held in registers at a time
template <int S>
__device__ __forceinline__ void sk_wload(const bf16* __restrict__ W, int ldw, int n0, int N, int k0,
                                         bf16x8 (&wf)[S]) {
  const int lane = threadIdx.x & 63, lq = lane & 15, g = lane >> 4;
  const bf16* wp = W + (size_t)min(n0 + lq, N - 1) * ldw + k0 + 8 * g;
#pragma unroll
  for (int u = 0; u < S; ++u) wf[u] = *reinterpret_cast<const bf16x8*>(wp + u * 32);
}
// Weights stored as FP8 E4M3 codes (1-4-3, bias 7, no infinities) with one fp32 scale per output
// row: the same operand positions, half the bytes per request; a fragment is up-cast to bf16
// (exact: 3 mantissa bits) right before its MFMA and the row scale multiplies the finished sum.
template <class WT> struct SkFrag { typedef bf16x8 type; };
template <class WT>
__device__ __forceinline__ float sk_wscale(const float* __restrict__ wscale, int n) {
  if constexpr (std::is_same<WT, bf16>::value) return 1.f;
  else return wscale[n];
}
template <> struct SkFrag<fp8> { typedef fp8x8 type; };
__device__ __forceinline__ bf16x8 sk_frag(const bf16x8& f) { return f; }
__device__ __forceinline__ bf16x8 sk_frag(const fp8x8& f) { return e4m3x8_to_bf16(f); }
template <int S>
__device__ __forceinline__ void sk_wload(const fp8* __restrict__ W, int ldw, int n0, int N, int k0, fp8x8 (&wf)[S]) {
  const int lane = threadIdx.x & 63, lq = lane & 15, g = lane >> 4;
  const fp8* wp = W + (size_t)min(n0 + lq, N - 1) * ldw + k0 + 8 * g;
#pragma unroll
  for (int u = 0; u < S; ++u) wf[u] = *reinterpret_cast<const fp8x8*>(wp + u * 32);
}
template <int S, bool TWO, class FR, class GetB>
__device__ __forceinline__ void sk_mma(const FR (&wf)[S], int k0, GetB&& getB, f32x4 (&acc)[2]) {
  const int g = (threadIdx.x & 63) >> 4;
#pragma unroll
  for (int u = 0; u < S; ++u) {
    const int k = k0 + u * 32 + 8 * g;
    const bf16x8 w = sk_frag(wf[u]);
    acc[0] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(w, getB(0, k), acc[0], 0, 0, 0);
    if (TWO) acc[1] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(w, getB(1, k), acc[1], 0, 0, 0);
  }
  mfma_settle(acc[0], acc[1]);
}
// steps kSkW .. STEPS - 1 of a long k range, kSkW at a time
template <int STEPS, bool TWO, class WT, class GetB>
__device__ __forceinline__ void sk_mma_tail(const WT* __restrict__ W, int ldw, int n0, int N, int k0,
                                            GetB&& getB, f32x4 (&acc)[2]) {
  if constexpr (STEPS > kSkW) {
    static_assert(STEPS % kSkW == 0, "long k ranges come in whole batches");
#pragma unroll 1
    for (int s0 = kSkW; s0 < STEPS; s0 += kSkW) {
      typename SkFrag<WT>::type wf[kSkW];
      sk_wload<kSkW>(W, ldw, n0, N, k0 + s0 * 32, wf);
      sk_mma<kSkW, TWO>(wf, k0 + s0 * 32, getB, acc);
    }
  }
}
__device__ __forceinline__ void sk_zero(f32x4 (&acc)[2]) {
  acc[0] = f32x4{0.f, 0.f, 0.f, 0.f};
  acc[1] = acc[0];
}

// Sum the 4 waves' partial tiles (fixed order) and hand every output (m, n local) to f.
// Thread t < 256 gets column n = t % 16 of rows m = t / 16 and t / 16 + 16 (callers prefetch what
// their f reads from memory for exactly these).
template <class F>
__device__ __forceinline__ void sk_reduce(const f32x4 (&acc)[2], float* red, int R, F&& f) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, lq = lane & 15, g = lane >> 4;
  if (wave < 4) {   // (a block may have more waves than the four that split K)
#pragma unroll
    for (int t = 0; t < 2; ++t)
#pragma unroll
      for (int r = 0; r < 4; ++r) red[(wave * 16 + 4 * g + r) * 33 + t * 16 + lq] = acc[t][r];
  }
  __syncthreads();
  for (int idx = threadIdx.x; idx < 16 * kSkRows && threadIdx.x < kSkThreads; idx += kSkThreads) {
    const int m = idx >> 4, n = idx & 15;
    if (m < R) {
      float v = red[(0 * 16 + n) * 33 + m];
      v += red[(1 * 16 + n) * 33 + m];
      v += red[(2 * 16 + n) * 33 + m];
      v += red[(3 * 16 + n) * 33 + m];
      f(m, n, v);
    }
  }
}

// Logit of the draft each row scores: D[i][j] = E[draft of row 16t+i] . h[16t+j] (wave t < 2)
// with the same instruction and k order as the vocabulary projection, hence bit-identical to
// the element the projection produces for that (row, column); the diagonal is kept.
// Two parts: sk_draft_fetch requests the embedding rows of the drafts (first the draft ids,
// then the rows: two round trips that run while the caller's prologue does), sk_draft_logit
// multiplies once the hidden rows are in LDS.
template <int PER, class WT = bf16>
struct SkDraft {
  static constexpr int kSteps = 2 * PER;   // d / 32
  typename SkFrag<WT>::type wf[kSteps];
  float scale;                             // row scale of the draft's embedding row (1 for bf16 weights)
  bool has;
};
// The draft of this lane's row (waves 0 and 1: row wave*16 + lane%16; others: -1).  Requested on its own,
// before the block's weight tile, so that waiting for it does not wait for the tile and the draft's
// embedding row is fetched while the tile streams in.
__device__ __forceinline__ int sk_draft_tok(int R, const int* __restrict__ row_draft) {
  const int wave = threadIdx.x >> 6;
  if (wave >= 2) return -1;
  return row_draft[min(wave * 16 + (int)(threadIdx.x & 15), R - 1)];
}
template <int PER, class WT>
__device__ __forceinline__ void sk_draft_fetch(SkDraft<PER, WT>& dr, int R, const WT* __restrict__ E, int V, int tok,
                                               const float* __restrict__ wscale) {
  constexpr int d = 64 * PER;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, lq = lane & 15, g = lane >> 4;
  dr.has = false;
  if (wave >= 2) return;
  const int row = wave * 16 + lq;
  dr.has = row < R && tok >= 0 && tok < V;
  dr.scale = wscale ? wscale[dr.has ? tok : 0] : 1.f;
  const WT* wp = E + (size_t)(dr.has ? tok : 0) * d + 8 * g;
#pragma unroll
  for (int s = 0; s < SkDraft<PER, WT>::kSteps; ++s)
    dr.wf[s] = *reinterpret_cast<const typename SkFrag<WT>::type*>(wp + s * 32);
}
template <int PER, class WT>
__device__ __forceinline__ void sk_draft_fetch(SkDraft<PER, WT>& dr, int R, const WT* __restrict__ E, int V,
                                               const int* __restrict__ row_draft, const float* __restrict__ wscale) {
  sk_draft_fetch<PER, WT>(dr, R, E, V, sk_draft_tok(R, row_draft), wscale);
}
template <int PER, class WT, class Out>
__device__ __forceinline__ void sk_draft_logit(const SkDraft<PER, WT>& dr, const bf16* hb, int R, Out&& out) {
  constexpr int d = 64 * PER, pitch = d + kSkPad;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, lq = lane & 15, g = lane >> 4;
  if (wave >= 2) return;
  const int row = wave * 16 + lq;
  f32x4 acc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
  for (int s = 0; s < SkDraft<PER, WT>::kSteps; ++s) {
    bf16x8 hf = *reinterpret_cast<const bf16x8*>(hb + row * pitch + s * 32 + 8 * g);
    acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(sk_frag(dr.wf[s]), hf, acc, 0, 0, 0);
  }
  mfma_settle(acc);
  // D[i][j]: this lane holds j = lq, i = 4g + r; diagonal i = j  <=>  g == lq/4, r = lq%4
  if (g == (lq >> 2) && row < R) {
    float v = 0.f;
#pragma unroll
    for (int r = 0; r < 4; ++r) if (r == (lq & 3)) v = acc[r];
    // (the row scale multiplies the sum exactly as the projection does for that column)
    out(row, dr.has ? v * dr.scale : kNegInf);
  }
}

// Row statistics of one 64-column vocabulary tile (16 columns per wave: acc of this wave,
// first column n0): per row the maximum, its lowest index, sum exp(z - max) and the number of
// logits above the row's draft logit zd[t] (row t*16 + lane%16); one record per row -> part.
__device__ __forceinline__ void sk_vocab_tile(const f32x4 (&acc)[2], int n0, int V, int R, const float (&zd_t)[2],
                                              float* red, float* __restrict__ part, int n_tiles, int tile,
                                              float* __restrict__ logits) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, lq = lane & 15, g = lane >> 4;
  // this lane: rows m = t*16 + lq, columns n0 + 4g + r
  // red: [4 waves][32 rows][4]: max, arg-max, sum-exp, count
#pragma unroll
  for (int t = 0; t < 2; ++t) {
    const int m = t * 16 + lq;
    const float zd = zd_t[t];
    float best = kNegInf;
    int besti = 0x7fffffff, cnt = 0;
#pragma unroll
    for (int r = 0; r < 4; ++r) {
      const int n = n0 + 4 * g + r;
      const float v = acc[t][r];
      if (n < V) {
        if (v > best) { best = v; besti = n; }
        cnt += (v > zd) ? 1 : 0;
        if (logits && m < R) logits[(size_t)m * V + n] = v;
      }
    }
#pragma unroll
    for (int o = 16; o <= 32; o <<= 1) {
      const float ob = __shfl_xor(best, o, 64);
      const int oi = __shfl_xor(besti, o, 64);
      if (ob > best || (ob == best && oi < besti)) { best = ob; besti = oi; }
      cnt += __shfl_xor(cnt, o, 64);
    }
    float se = 0.f;
#pragma unroll
    for (int r = 0; r < 4; ++r)
      if (n0 + 4 * g + r < V) se += __expf(acc[t][r] - best);
    se += __shfl_xor(se, 16, 64);
    se += __shfl_xor(se, 32, 64);
    if (g == 0) {
      float* p = red + (wave * 32 + m) * 4;
      p[0] = best; p[1] = __int_as_float(besti); p[2] = se; p[3] = __int_as_float(cnt);
    }
  }
  __syncthreads();
  if (threadIdx.x < kSkRows && (int)threadIdx.x < R) {
    const int m = threadIdx.x;
    float best = kNegInf, tot = 0.f;
    int besti = 0x7fffffff, cnt = 0;
#pragma unroll
    for (int w = 0; w < 4; ++w) {
      const float* p = red + (w * 32 + m) * 4;
      const int bi = __float_as_int(p[1]);
      if (p[0] > best || (p[0] == best && bi < besti)) { best = p[0]; besti = bi; }
      cnt += __float_as_int(p[3]);
    }
#pragma unroll
    for (int w = 0; w < 4; ++w) {
      const float* p = red + (w * 32 + m) * 4;
      if (p[0] > kNegInf) tot += p[2] * __expf(p[0] - best);
    }
    f32x4 rec = {best, __int_as_float(besti), tot, __int_as_float(cnt)};
    *reinterpret_cast<f32x4*>(part + ((size_t)m * n_tiles + tile) * kPartF) = rec;
  }
}

}  // namespace sd
