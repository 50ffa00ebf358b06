// Fused kernels for passes of at most 32 rows (single-sequence verification, Sec. 2).
//
// With so few rows a decoder pass is a chain of weight-streaming products whose cost is the
// number of dependent kernels, not their arithmetic.  Each kernel here is one projection with
// everything that precedes it folded into its prologue, recomputed redundantly by every block
// (the whole activation block is at most 32 x 1024 values):
//   qkv      : [embedding | LayerNorm of the previous sum]            -> Q, K/V append
//   attn_o   : residual LayerNorm, attention of every head, O-projection -> new residual sum
//   cross_q  : LayerNorm                                               -> cross-attention Q
//   (attn_o again with the cross K/V)
//   ffn1     : LayerNorm, W1, ReLU                                     -> hidden
//   ffn2     : residual LayerNorm, W2                                  -> new residual sum
//   vocab    : LayerNorm, tied output projection, row statistics per 64-column tile
// A block owns 16 output columns; its 4 waves split K, every wave issues all its weight loads
// before the first MFMA (one memory round trip per kernel), and the 4 partial tiles are summed
// through LDS in a fixed order.  MFMA 16x16x32: A = 16 weight rows, B = up to 2 x 16 activation
// rows, so D[n][m]: lane holds row m = lane%16, columns n = 4*(lane/16) + r.
#include "attn_core.h"

namespace sd {

constexpr int kSkThreads = 256;
constexpr int kSkRows = 32;          // activation rows a block can hold (2 MFMA column tiles)
constexpr int kSkPad = 8;            // bf16 padding of an activation row in LDS (bank spread)

// LDS carve-up (dynamic): hb bf16 [32][d + 8] | hown f32 [32][16] | red f32 [4][16][33] | Vs
template <int PER>
struct SkLds {
  static constexpr int d = 64 * PER;
  static constexpr int kPitch = d + kSkPad;
  static constexpr size_t kHb = (size_t)kSkRows * kPitch * 2;
  static constexpr size_t kOwn = (size_t)kSkRows * 16 * 4;
  static constexpr size_t kRed = (size_t)4 * 16 * 33 * 4;
  static constexpr size_t kVs = (size_t)4 * 32 * kVtPitch * 2;
  static constexpr size_t kBytes = kHb + kOwn + kRed + kVs;
  bf16* hb; float* hown; float* red; bf16 (*vs)[32][kVtPitch];
  __device__ explicit SkLds(char* base) {
    hb = reinterpret_cast<bf16*>(base);
    hown = reinterpret_cast<float*>(base + kHb);
    red = reinterpret_cast<float*>(base + kHb + kOwn);
    vs = reinterpret_cast<bf16 (*)[32][kVtPitch]>(base + kHb + kOwn + kRed);
  }
};

// Hidden state of the R rows = what `src` describes; bf16 copy of all columns -> hb (rows
// R .. nrows-1 zero), fp32 copy of columns [n0, n0 + 16) -> hown (for residual adds).
// A wave takes rows wave, wave + 4, ...; it requests the data of up to four of them (and the
// LayerNorm parameters, once) before it reduces any, so the prologue costs one memory round
// trip however many rows there are.
template <int PER>
__device__ __forceinline__ void sk_hidden(const SkSrc& s, int R, int nrows, bf16* hb, float* hown, int n0,
                                          bool want_hb) {
  constexpr int d = 64 * PER, pitch = d + kSkPad, RU = 4;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  float gg[PER], bb[PER];
  if (s.mode == 2) {
#pragma unroll
    for (int i = 0; i < PER; ++i) { gg[i] = (float)s.g[i * 64 + lane]; bb[i] = (float)s.b[i * 64 + lane]; }
  }
  for (int base = wave; base < nrows; base += 4 * RU) {
    float v[RU][PER];
    if (s.mode == 0) {
      int tok[RU], pos[RU];
#pragma unroll
      for (int u = 0; u < RU; ++u) {
        const int r = min(base + 4 * u, R - 1);
        tok[u] = s.tok[r]; pos[u] = s.pos[r];
      }
      const float sc = sqrtf((float)d);
#pragma unroll
      for (int u = 0; u < RU; ++u) {
        const bf16* e = s.E + (size_t)tok[u] * d;
        const float* p = s.pe + (size_t)pos[u] * d;
#pragma unroll
        for (int i = 0; i < PER; ++i) v[u][i] = (float)e[i * 64 + lane] * sc + p[i * 64 + lane];
      }
    } else {
#pragma unroll
      for (int u = 0; u < RU; ++u) {
        const int r = min(base + 4 * u, R - 1);
#pragma unroll
        for (int i = 0; i < PER; ++i) v[u][i] = s.xs[(size_t)r * d + i * 64 + lane];
      }
      if (s.mode == 2) {
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
          rstd[u] = 1.0f / sqrtf(wave_sum(q) / (float)d + 1e-5f);
        }
#pragma unroll
        for (int u = 0; u < RU; ++u)
#pragma unroll
          for (int i = 0; i < PER; ++i) v[u][i] = (v[u][i] - mean[u]) * rstd[u] * gg[i] + bb[i];
      }
    }
#pragma unroll
    for (int u = 0; u < RU; ++u) {
      const int r = base + 4 * u;
      if (r < nrows) {
        const bool real = r < R;
#pragma unroll
        for (int i = 0; i < PER; ++i) {
          const int c = i * 64 + lane;
          const float val = real ? v[u][i] : 0.f;
          if (want_hb) hb[r * pitch + c] = (bf16)val;
          if (c >= n0 && c < n0 + 16) hown[r * 16 + c - n0] = val;
        }
      }
    }
  }
}

// Weight operands of this wave: rows n0 + lane%16 of W, k range [k0, k0 + 32*S).  sk_wload only
// issues the loads -- kernels call it first thing, so the weights travel while the prologue
// (LayerNorm, attention) runs; sk_mma consumes them:
//   acc[t] += W[n0 + i][k] . B_t[j][k],  getB(t, k) = 8 bf16 of activation row t*16 + lane%16 at k.
// Step counts and the second row tile are compile-time, so the MFMA sequence is straight-line.
constexpr int kSkW = 16;   // most steps held in registers at a time
template <int S>
__device__ __forceinline__ void sk_wload(const bf16* __restrict__ W, int ldw, int n0, int N, int k0,
                                         bf16x8 (&wf)[S]) {
  const int lane = threadIdx.x & 63, lq = lane & 15, g = lane >> 4;
  const bf16* wp = W + (size_t)min(n0 + lq, N - 1) * ldw + k0 + 8 * g;
#pragma unroll
  for (int u = 0; u < S; ++u) wf[u] = *reinterpret_cast<const bf16x8*>(wp + u * 32);
}
template <int S, bool TWO, class GetB>
__device__ __forceinline__ void sk_mma(const bf16x8 (&wf)[S], int k0, GetB&& getB, f32x4 (&acc)[2]) {
  const int g = (threadIdx.x & 63) >> 4;
#pragma unroll
  for (int u = 0; u < S; ++u) {
    const int k = k0 + u * 32 + 8 * g;
    acc[0] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(wf[u], getB(0, k), acc[0], 0, 0, 0);
    if (TWO) acc[1] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(wf[u], getB(1, k), acc[1], 0, 0, 0);
  }
}
// steps kSkW .. STEPS - 1 of a long k range, kSkW at a time
template <int STEPS, bool TWO, class GetB>
__device__ __forceinline__ void sk_mma_tail(const bf16* __restrict__ W, int ldw, int n0, int N, int k0,
                                            GetB&& getB, f32x4 (&acc)[2]) {
  if constexpr (STEPS > kSkW) {
    static_assert(STEPS % kSkW == 0, "long k ranges come in whole batches");
#pragma unroll 1
    for (int s0 = kSkW; s0 < STEPS; s0 += kSkW) {
      bf16x8 wf[kSkW];
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
template <class F>
__device__ __forceinline__ void sk_reduce(const f32x4 (&acc)[2], float* red, int R, F&& f) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, lq = lane & 15, g = lane >> 4;
#pragma unroll
  for (int t = 0; t < 2; ++t)
#pragma unroll
    for (int r = 0; r < 4; ++r) red[(wave * 16 + 4 * g + r) * 33 + t * 16 + lq] = acc[t][r];
  __syncthreads();
  for (int idx = threadIdx.x; idx < 16 * kSkRows; idx += kSkThreads) {
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

// ------------------------------------------------------------------------------------ qkv
template <int PER, bool TWO>
__global__ __launch_bounds__(kSkThreads) void sk_qkv_kernel(SkSrc src, int R, const bf16* __restrict__ W,
                                                            const bf16* __restrict__ bias, bf16* __restrict__ q,
                                                            bf16* __restrict__ kc, bf16* __restrict__ vc,
                                                            const int* __restrict__ row_b,
                                                            const int* __restrict__ row_pos, int H, int Lcap) {
  extern __shared__ __attribute__((aligned(16))) char sk_smem[];
  SkLds<PER> L(sk_smem);
  constexpr int d = 64 * PER, pitch = d + kSkPad;
  const int n0 = blockIdx.x * 16, wave = threadIdx.x >> 6, lq = threadIdx.x & 15;
  constexpr int steps = d / 128;
  const int k0 = wave * (d / 4);
  bf16x8 wf[steps];
  sk_wload<steps>(W, d, n0, 3 * d, k0, wf);
  sk_hidden<PER>(src, R, TWO ? 32 : 16, L.hb, L.hown, -64, true);
  __syncthreads();
  f32x4 acc[2];
  sk_zero(acc);
  const bf16* hb = L.hb;
  sk_mma<steps, TWO>(wf, k0,
         [&](int t, int k) { return *reinterpret_cast<const bf16x8*>(hb + (t * 16 + lq) * pitch + k); }, acc);
  sk_reduce(acc, L.red, R, [&](int m, int nl, float v) {
    const int n = n0 + nl;
    v += (float)bias[n];
    const int part = n / d, c = n - part * d;
    if (part == 0) { q[(size_t)m * d + c] = (bf16)v; return; }
    const int b = row_b[m];
    if (b < 0) return;
    bf16* cache = (part == 1) ? kc : vc;
    cache[(((size_t)b * H + (c >> 6)) * Lcap + row_pos[m]) * kHeadDim + (c & 63)] = (bf16)v;
  });
}

// ------------------------------------------------------------------------------------ attention + O
// resid: hidden state the sublayer started from (its own 16 columns are added back).
template <int PER, bool VBLK, bool TWO>
__global__ __launch_bounds__(kSkThreads) void sk_attn_o_kernel(SkSrc resid, int R, AttnArgs a,
                                                               const bf16* __restrict__ W,
                                                               const bf16* __restrict__ bias,
                                                               float* __restrict__ xs_out) {
  extern __shared__ __attribute__((aligned(16))) char sk_smem[];
  SkLds<PER> L(sk_smem);
  constexpr int d = 64 * PER, pitch = d + kSkPad;
  const int n0 = blockIdx.x * 16, lane = threadIdx.x & 63, wave = threadIdx.x >> 6, lq = lane & 15, g = lane >> 4;
  constexpr int steps = d / 128;
  const int k0 = wave * (d / 4);
  bf16x8 wf[steps];
  sk_wload<steps>(W, d, n0, d, k0, wf);
  sk_hidden<PER>(resid, R, TWO ? 32 : 16, L.hb, L.hown, n0, false);
  // attention output of every (sequence, head) pair -> hb (bf16 [32][d]); rows >= R zero
  for (int idx = threadIdx.x; idx < (TWO ? 32 : 16) * pitch / 8; idx += kSkThreads)
    reinterpret_cast<uint4*>(L.hb)[idx] = make_uint4(0, 0, 0, 0);
  __syncthreads();
  for (int p = wave; p < a.B * a.H; p += 4) {
    const int b = p / a.H, h = p - b * a.H;
    constexpr int NQT = TWO ? 2 : 1;   // at most 16 rows in all: one query tile
    const int nq = min(a.q_count ? a.q_count[b] : a.T, 16 * NQT);
    float mrun[NQT], lrun[NQT];
    f32x4 oacc[NQT][4];
    attn_wave<NQT, VBLK>(a, b, h, 0, nq, 0, 1, L.vs[wave], mrun, lrun, oacc);
#pragma unroll
    for (int qt = 0; qt < NQT; ++qt) {
      const int qi = qt * 16 + lq;
      if (qi < nq) {
        const float inv = lrun[qt] > 0.f ? 1.f / lrun[qt] : 0.f;
        bf16* op = L.hb + (b * a.T + qi) * pitch + h * kHeadDim;
#pragma unroll
        for (int et = 0; et < 4; ++et)
#pragma unroll
          for (int r = 0; r < 4; ++r) op[et * 16 + 4 * g + r] = (bf16)(oacc[qt][et][r] * inv);
      }
    }
  }
  __syncthreads();
  f32x4 acc[2];
  sk_zero(acc);
  const bf16* hb = L.hb;
  sk_mma<steps, TWO>(wf, k0,
         [&](int t, int k) { return *reinterpret_cast<const bf16x8*>(hb + (t * 16 + lq) * pitch + k); }, acc);
  const float* hown = L.hown;
  sk_reduce(acc, L.red, R, [&](int m, int nl, float v) {
    xs_out[(size_t)m * d + n0 + nl] = v + (float)bias[n0 + nl] + hown[m * 16 + nl];
  });
}

// ------------------------------------------------------------------------------------ plain projection
// out = act(hidden W^T + bias) as bf16 [R][N] (cross-attention Q, FFN1)
template <int PER, bool TWO>
__global__ __launch_bounds__(kSkThreads) void sk_proj_kernel(SkSrc src, int R, const bf16* __restrict__ W, int N,
                                                             const bf16* __restrict__ bias, bf16* __restrict__ out,
                                                             int relu) {
  extern __shared__ __attribute__((aligned(16))) char sk_smem[];
  SkLds<PER> L(sk_smem);
  constexpr int d = 64 * PER, pitch = d + kSkPad;
  const int n0 = blockIdx.x * 16, wave = threadIdx.x >> 6, lq = threadIdx.x & 15;
  constexpr int steps = d / 128;
  const int k0 = wave * (d / 4);
  bf16x8 wf[steps];
  sk_wload<steps>(W, d, n0, N, k0, wf);
  sk_hidden<PER>(src, R, TWO ? 32 : 16, L.hb, L.hown, -64, true);
  __syncthreads();
  f32x4 acc[2];
  sk_zero(acc);
  const bf16* hb = L.hb;
  sk_mma<steps, TWO>(wf, k0,
         [&](int t, int k) { return *reinterpret_cast<const bf16x8*>(hb + (t * 16 + lq) * pitch + k); }, acc);
  sk_reduce(acc, L.red, R, [&](int m, int nl, float v) {
    if (n0 + nl < N) {
      v += (float)bias[n0 + nl];
      if (relu) v = fmaxf(v, 0.f);
      out[(size_t)m * N + n0 + nl] = (bf16)v;
    }
  });
}

// ------------------------------------------------------------------------------------ FFN2
// xs_out = hidden(resid) + hid W2^T + bias; hid bf16 [R][F] is read straight from memory
template <int PER, int FS, bool TWO>   // FS = F / 128 = k steps per wave
__global__ __launch_bounds__(kSkThreads) void sk_ffn2_kernel(SkSrc resid, int R, const bf16* __restrict__ hid,
                                                             const bf16* __restrict__ W,
                                                             const bf16* __restrict__ bias,
                                                             float* __restrict__ xs_out) {
  extern __shared__ __attribute__((aligned(16))) char sk_smem[];
  SkLds<PER> L(sk_smem);
  constexpr int d = 64 * PER, F = 128 * FS, S1 = FS < kSkW ? FS : kSkW;
  const int n0 = blockIdx.x * 16, wave = threadIdx.x >> 6, lq = threadIdx.x & 15, g = (threadIdx.x & 63) >> 4;
  const int k0 = wave * (F / 4);
  bf16x8 wf[S1], hf[S1];
  sk_wload<S1>(W, F, n0, d, k0, wf);
  // first-tile activations of the same k range, straight from memory (same operand layout)
  {
    const bf16* hp = hid + (size_t)min(lq, R - 1) * F + k0 + 8 * g;
#pragma unroll
    for (int u = 0; u < S1; ++u) hf[u] = *reinterpret_cast<const bf16x8*>(hp + u * 32);
  }
  sk_hidden<PER>(resid, R, TWO ? 32 : 16, L.hb, L.hown, n0, false);
  f32x4 acc[2];
  sk_zero(acc);
  auto getB = [&](int t, int k) {
    return *reinterpret_cast<const bf16x8*>(hid + (size_t)min(t * 16 + lq, R - 1) * F + k);
  };
#pragma unroll
  for (int u = 0; u < S1; ++u) {
    acc[0] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(wf[u], hf[u], acc[0], 0, 0, 0);
    if (TWO) acc[1] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(wf[u], getB(1, k0 + u * 32 + 8 * g), acc[1], 0, 0, 0);
  }
  sk_mma_tail<FS, TWO>(W, F, n0, d, k0, getB, acc);
  __syncthreads();
  const float* hown = L.hown;
  sk_reduce(acc, L.red, R, [&](int m, int nl, float v) {
    xs_out[(size_t)m * d + n0 + nl] = v + (float)bias[n0 + nl] + hown[m * 16 + nl];
  });
}

// ------------------------------------------------------------------------------------ vocabulary
// Draft logits first (one block, one wave per 16 rows): D[i][j] = E[draft of row 16t+i] . h[16t+j]
// with the same instruction and k order as the projection below, hence bit-identical to the
// element the projection produces for that (row, column); the diagonal is kept.
template <int PER>
__global__ __launch_bounds__(kSkThreads) void sk_draft_logit_kernel(SkSrc src, int R, const bf16* __restrict__ E,
                                                                    int V, const int* __restrict__ row_draft,
                                                                    float* __restrict__ zd_out) {
  extern __shared__ __attribute__((aligned(16))) char sk_smem[];
  SkLds<PER> L(sk_smem);
  constexpr int d = 64 * PER, pitch = d + kSkPad;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, lq = lane & 15, g = lane >> 4;
  sk_hidden<PER>(src, R, R > 16 ? 32 : 16, L.hb, L.hown, -64, true);
  __syncthreads();
  if (wave >= 2) return;
  const int t = wave;
  const int row = t * 16 + lq;
  const int tok = row < R ? row_draft[row] : -1;
  const bool has = tok >= 0 && tok < V;
  const bf16* wp = E + (size_t)(has ? tok : 0) * d + 8 * g;
  f32x4 acc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll 8
  for (int s = 0; s < d / 32; ++s) {
    bf16x8 wf = *reinterpret_cast<const bf16x8*>(wp + s * 32);
    bf16x8 hf = *reinterpret_cast<const bf16x8*>(L.hb + row * pitch + s * 32 + 8 * g);
    acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(wf, hf, acc, 0, 0, 0);
  }
  // D[i][j]: this lane holds j = lq, i = 4g + r; diagonal i = j  <=>  g == lq/4, r = lq%4
  if (g == (lq >> 2) && row < R) {
    float v = 0.f;
#pragma unroll
    for (int r = 0; r < 4; ++r) if (r == (lq & 3)) v = acc[r];
    zd_out[row] = has ? v : kNegInf;
  }
}

// One block = 64 vocabulary columns (16 per wave, whole K per wave), one partial record per row.
template <int PER, bool TWO>
__global__ __launch_bounds__(kSkThreads) void sk_vocab_kernel(SkSrc src, int R, const bf16* __restrict__ E, int V,
                                                              const float* __restrict__ zd_row,
                                                              float* __restrict__ part, int n_tiles,
                                                              float* __restrict__ logits) {
  extern __shared__ __attribute__((aligned(16))) char sk_smem[];
  SkLds<PER> L(sk_smem);
  constexpr int d = 64 * PER, pitch = d + kSkPad;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, lq = lane & 15, g = lane >> 4;
  const int n0 = blockIdx.x * 64 + wave * 16;
  constexpr int steps = d / 32, S1 = steps < kSkW ? steps : kSkW;
  bf16x8 wf[S1];
  sk_wload<S1>(E, d, n0, V, 0, wf);
  sk_hidden<PER>(src, R, TWO ? 32 : 16, L.hb, L.hown, -64, true);
  __syncthreads();
  f32x4 acc[2];
  sk_zero(acc);
  const bf16* hb = L.hb;
  auto getB = [&](int t, int k) { return *reinterpret_cast<const bf16x8*>(hb + (t * 16 + lq) * pitch + k); };
  sk_mma<S1, TWO>(wf, 0, getB, acc);
  sk_mma_tail<steps, TWO>(E, d, n0, V, 0, getB, acc);
  // this lane: rows m = t*16 + lq, columns n0 + 4g + r
  float* red = L.red;   // [4 waves][32 rows][4]: max, arg-max, sum-exp, count
#pragma unroll
  for (int t = 0; t < 2; ++t) {
    const int m = t * 16 + lq;
    const float zd = m < R ? zd_row[m] : kNegInf;
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
    *reinterpret_cast<f32x4*>(part + ((size_t)m * n_tiles + blockIdx.x) * kPartF) = rec;
  }
}

// ------------------------------------------------------------------------------------ launchers
template <int PER, class K>
static hipError_t sk_attr(K kernel) {
  return hipFuncSetAttribute(reinterpret_cast<const void*>(kernel), hipFuncAttributeMaxDynamicSharedMemorySize,
                             (int)SkLds<PER>::kBytes);
}

bool skinny_supported(int d, int F) {
  return (d == 128 || d == 512 || d == 1024) && (F == 256 || F == 2048 || F == 4096);
}

#define SK_DISPATCH(d, CALL)                      \
  switch ((d) / 64) {                             \
    case 2: { constexpr int PER = 2; CALL; } break;   \
    case 8: { constexpr int PER = 8; CALL; } break;   \
    case 16: { constexpr int PER = 16; CALL; } break; \
    default: return hipErrorInvalidValue;         \
  }
#define SK_ROWS(R, CALL)                                        \
  if ((R) > 16) { constexpr bool TWO = true; CALL; }            \
  else { constexpr bool TWO = false; CALL; }
#define SK_FFN(F, CALL)                               \
  switch ((F) / 128) {                                \
    case 2: { constexpr int FS = 2; CALL; } break;    \
    case 16: { constexpr int FS = 16; CALL; } break;  \
    case 32: { constexpr int FS = 32; CALL; } break;  \
    default: return hipErrorInvalidValue;             \
  }

template <int PER, bool TWO>
static hipError_t sk_init_rows() {
  hipError_t e;
  if ((e = sk_attr<PER>(sk_qkv_kernel<PER, TWO>)) != hipSuccess) return e;
  if ((e = sk_attr<PER>(sk_attn_o_kernel<PER, false, TWO>)) != hipSuccess) return e;
  if ((e = sk_attr<PER>(sk_attn_o_kernel<PER, true, TWO>)) != hipSuccess) return e;
  if ((e = sk_attr<PER>(sk_proj_kernel<PER, TWO>)) != hipSuccess) return e;
  if ((e = sk_attr<PER>(sk_ffn2_kernel<PER, 2, TWO>)) != hipSuccess) return e;
  if ((e = sk_attr<PER>(sk_ffn2_kernel<PER, 16, TWO>)) != hipSuccess) return e;
  if ((e = sk_attr<PER>(sk_ffn2_kernel<PER, 32, TWO>)) != hipSuccess) return e;
  if ((e = sk_attr<PER>(sk_vocab_kernel<PER, TWO>)) != hipSuccess) return e;
  return hipSuccess;
}

hipError_t skinny_init(int d) {
  hipError_t e = hipSuccess;
  SK_DISPATCH(d, {
    if ((e = sk_init_rows<PER, false>()) != hipSuccess) return e;
    if ((e = sk_init_rows<PER, true>()) != hipSuccess) return e;
    if ((e = sk_attr<PER>(sk_draft_logit_kernel<PER>)) != hipSuccess) return e;
  });
  return e;
}

hipError_t skinny_qkv(hipStream_t st, const SkSrc& src, int R, int d, const bf16* W, const bf16* bias, bf16* q,
                      bf16* kc, bf16* vc, const int* row_b, const int* row_pos, int H, int Lcap) {
  SK_DISPATCH(d, SK_ROWS(R, hipLaunchKernelGGL((sk_qkv_kernel<PER, TWO>), dim3(3 * d / 16), dim3(kSkThreads),
                                               SkLds<PER>::kBytes, st, src, R, W, bias, q, kc, vc, row_b, row_pos,
                                               H, Lcap)));
  return hipGetLastError();
}
hipError_t skinny_attn_o(hipStream_t st, const SkSrc& resid, int R, int d, const AttnArgs& a, const bf16* W,
                         const bf16* bias, float* xs_out) {
  if (a.v_blocked) {
    SK_DISPATCH(d, SK_ROWS(R, hipLaunchKernelGGL((sk_attn_o_kernel<PER, true, TWO>), dim3(d / 16), dim3(kSkThreads),
                                                 SkLds<PER>::kBytes, st, resid, R, a, W, bias, xs_out)));
  } else {
    SK_DISPATCH(d, SK_ROWS(R, hipLaunchKernelGGL((sk_attn_o_kernel<PER, false, TWO>), dim3(d / 16), dim3(kSkThreads),
                                                 SkLds<PER>::kBytes, st, resid, R, a, W, bias, xs_out)));
  }
  return hipGetLastError();
}
hipError_t skinny_proj(hipStream_t st, const SkSrc& src, int R, int d, const bf16* W, int N, const bf16* bias,
                       bf16* out, bool relu) {
  SK_DISPATCH(d, SK_ROWS(R, hipLaunchKernelGGL((sk_proj_kernel<PER, TWO>), dim3((N + 15) / 16), dim3(kSkThreads),
                                               SkLds<PER>::kBytes, st, src, R, W, N, bias, out, relu ? 1 : 0)));
  return hipGetLastError();
}
hipError_t skinny_ffn2(hipStream_t st, const SkSrc& resid, int R, int d, const bf16* hid, int F, const bf16* W,
                       const bf16* bias, float* xs_out) {
  SK_DISPATCH(d, SK_FFN(F, SK_ROWS(R, hipLaunchKernelGGL((sk_ffn2_kernel<PER, FS, TWO>), dim3(d / 16),
                                                         dim3(kSkThreads), SkLds<PER>::kBytes, st, resid, R, hid, W,
                                                         bias, xs_out))));
  return hipGetLastError();
}
hipError_t skinny_vocab(hipStream_t st, const SkSrc& src, int R, int d, const bf16* E, int V, const int* row_draft,
                        float* zd_row, float* part, float* logits) {
  const int n_tiles = (V + 63) / 64;
  SK_DISPATCH(d, {
    hipLaunchKernelGGL(sk_draft_logit_kernel<PER>, dim3(1), dim3(kSkThreads), SkLds<PER>::kBytes, st, src, R, E, V,
                       row_draft, zd_row);
    SK_ROWS(R, hipLaunchKernelGGL((sk_vocab_kernel<PER, TWO>), dim3(n_tiles), dim3(kSkThreads), SkLds<PER>::kBytes,
                                  st, src, R, E, V, zd_row, part, n_tiles, logits));
  });
  return hipGetLastError();
}

}  // namespace sd
