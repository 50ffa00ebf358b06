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
//
// Every kernel exists for two weight types WT: bf16, and FP8 E4M3 codes with one fp32 scale per
// output row (wscale; half the streamed bytes).  The codes become bf16 operands in registers,
// the scale multiplies the finished fp32 sum before the bias: y = s_n * (sum_k q_nk h_k) + b_n.
#include "skinny_core.h"

namespace sd {


// ------------------------------------------------------------------------------------ qkv
template <int PER, bool TWO, class WT>
__global__ __launch_bounds__(kSkThreads) void sk_qkv_kernel(SkSrc src, int R, const WT* __restrict__ W,
                                                            const float* __restrict__ wscale,
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
  typename SkFrag<WT>::type wf[steps];
  sk_wload<steps>(W, d, n0, 3 * d, k0, wf);
  // what the epilogue reads from memory for this thread's outputs (sk_reduce: column
  // threadIdx % 16, rows threadIdx / 16 and + 16) is requested now, not after the product
  const bf16 bias_n = bias[n0 + (threadIdx.x & 15)];
  const float ws_n = sk_wscale<WT>(wscale, n0 + (threadIdx.x & 15));
  int rb[2], rp[2];
#pragma unroll
  for (int t = 0; t < 2; ++t) {
    const int m = min((int)(threadIdx.x >> 4) + 16 * t, R - 1);
    rb[t] = row_b[m]; rp[t] = row_pos[m];
  }
  sk_hidden<PER>(src, R, TWO ? 32 : 16, L.hb, L.hown, -64, true);
  __syncthreads();
  f32x4 acc[2];
  sk_zero(acc);
  const bf16* hb = L.hb;
  sk_mma<steps, TWO>(wf, k0,
         [&](int t, int k) { return *reinterpret_cast<const bf16x8*>(hb + (t * 16 + lq) * pitch + k); }, acc);
  sk_reduce(acc, L.red, R, [&](int m, int nl, float v) {
    const int n = n0 + nl;
    v = v * ws_n + (float)bias_n;
    const int part = n / d, c = n - part * d;
    if (part == 0) { q[(size_t)m * d + c] = (bf16)v; return; }
    const int b = rb[m >> 4];
    if (b < 0) return;
    bf16* cache = (part == 1) ? kc : vc;
    cache[(((size_t)b * H + (c >> 6)) * Lcap + rp[m >> 4]) * kHeadDim + (c & 63)] = (bf16)v;
  });
}

// ------------------------------------------------------------------------------------ attention + O
// resid: hidden state the sublayer started from (its own 16 columns are added back).
template <int PER, bool VBLK, bool TWO, class WT, bool KV8 = false>
__global__ __launch_bounds__(64 * kSkAttnWaves) void sk_attn_o_kernel(SkSrc resid, int R, AttnArgs a,
                                                                      const WT* __restrict__ W,
                                                                      const float* __restrict__ wscale,
                                                                      const bf16* __restrict__ bias,
                                                                      float* __restrict__ xs_out) {
  extern __shared__ __attribute__((aligned(16))) char sk_smem[];
  SkLds<PER> L(sk_smem);
  constexpr int d = 64 * PER, pitch = d + kSkPad, steps = d / 128;
  const int n0 = blockIdx.x * 16, lane = threadIdx.x & 63, wave = threadIdx.x >> 6, lq = lane & 15, g = lane >> 4;
  const bool kwave = wave < 4;                 // the four waves that split K of the O-projection
  const int k0 = (wave & 3) * (d / 4);
  typename SkFrag<WT>::type wf[steps];
  // hb receives the attention output of every (sequence, head) pair.  Its rows beyond R are
  // left as they are: an activation row only feeds its own output row, and those are dropped.
  // the block's 16 columns of the sublayer's input (for the residual add) are requested now
  // (rows wave, wave + 8, ... of every wave) and normalised after the attention, whose own
  // requests travel at the same time
  SkHidden<PER, false, TWO ? 4 : 2, kSkAttnWaves> hs;
  if (kwave) sk_wload<steps>(W, d, n0, d, k0, wf);
  const bf16 bias_n = bias[n0 + (threadIdx.x & 15)];   // for the epilogue (sk_reduce: column threadIdx % 16)
  const float ws_n = sk_wscale<WT>(wscale, n0 + (threadIdx.x & 15));
  hs.params(resid);
  hs.load(resid, R, wave);
  // One pair per wave: eight pairs are in flight at once.
  for (int p = wave; p < a.B * a.H; p += kSkAttnWaves) {
    const int b = p / a.H, h = p - b * a.H;
    constexpr int NQT = TWO ? 2 : 1;   // at most 16 rows in all: one query tile
    int nq = -1;   // min(query count of b, 16 * NQT): read inside, after the first key / value requests
    float mrun[NQT], lrun[NQT];
    f32x4 oacc[NQT][4];
    attn_wave<NQT, VBLK, false, false, KV8, false>(a, b, h, 0, nq, 0, 1, L.vs[wave], mrun, lrun, oacc);
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
  hs.finish(resid, R, TWO ? 32 : 16, wave, L.hb, L.hown, n0, false, -64);
  __syncthreads();
  f32x4 acc[2];
  sk_zero(acc);
  const bf16* hb = L.hb;
  if (kwave)
    sk_mma<steps, TWO>(wf, k0,
           [&](int t, int k) { return *reinterpret_cast<const bf16x8*>(hb + (t * 16 + lq) * pitch + k); }, acc);
  const float* hown = L.hown;
  sk_reduce(acc, L.red, R, [&](int m, int nl, float v) {
    xs_out[(size_t)m * d + n0 + nl] = v * ws_n + (float)bias_n + hown[m * 16 + nl];
  });
}

// ------------------------------------------------------------------------------------ plain projection
// out = act(hidden W^T + bias) as bf16 [R][N] (cross-attention Q, FFN1)
template <int PER, bool TWO, class WT>
__global__ __launch_bounds__(kSkThreads) void sk_proj_kernel(SkSrc src, int R, const WT* __restrict__ W,
                                                             const float* __restrict__ wscale, int N,
                                                             const bf16* __restrict__ bias, bf16* __restrict__ out,
                                                             int relu) {
  extern __shared__ __attribute__((aligned(16))) char sk_smem[];
  SkLds<PER> L(sk_smem);
  constexpr int d = 64 * PER, pitch = d + kSkPad;
  const int n0 = blockIdx.x * 16, wave = threadIdx.x >> 6, lq = threadIdx.x & 15;
  constexpr int steps = d / 128;
  const int k0 = wave * (d / 4);
  typename SkFrag<WT>::type wf[steps];
  sk_wload<steps>(W, d, n0, N, k0, wf);
  const bf16 bias_n = bias[min(n0 + (int)(threadIdx.x & 15), N - 1)];   // for the epilogue (column threadIdx % 16)
  const float ws_n = sk_wscale<WT>(wscale, min(n0 + (int)(threadIdx.x & 15), N - 1));
  sk_hidden<PER>(src, R, TWO ? 32 : 16, L.hb, L.hown, -64, true);
  __syncthreads();
  f32x4 acc[2];
  sk_zero(acc);
  const bf16* hb = L.hb;
  sk_mma<steps, TWO>(wf, k0,
         [&](int t, int k) { return *reinterpret_cast<const bf16x8*>(hb + (t * 16 + lq) * pitch + k); }, acc);
  sk_reduce(acc, L.red, R, [&](int m, int nl, float v) {
    if (n0 + nl < N) {
      v = v * ws_n + (float)bias_n;
      if (relu) v = fmaxf(v, 0.f);
      out[(size_t)m * N + n0 + nl] = (bf16)v;
    }
  });
}

// ------------------------------------------------------------------------------------ FFN2
// xs_out = hidden(resid) + hid W2^T + bias, hid bf16 [R][F].
// STAGED (whenever it fits: everything but 32 rows of F = 4096): the R rows of hid go to LDS
// first, one global->LDS request of 1 KB per wave, row and 512 columns -- R * F / 512 requests per
// block instead of one 16-byte register load per wave, k step and row tile; the products then read
// both row tiles from LDS.  Otherwise the first tile's operands come straight from memory into
// registers and the second tile's inside the loop.
template <int FS, bool TWO>
struct SkFfn2Lds {
  static constexpr int F = 128 * FS, kPitch = F + kSkPad, kRowsMax = TWO ? 32 : 16;
  static constexpr size_t kHid = (size_t)kRowsMax * kPitch * 2;
  static constexpr size_t kOwn = (size_t)2 * kSkRows * 16 * 4, kRed = (size_t)4 * 16 * 33 * 4;
  static constexpr size_t kBytes = kHid + kOwn + kRed;
  static constexpr bool kStaged = kBytes <= 150 * 1024 && F % 512 == 0;   // whole 512-column requests
};
template <int PER, int FS, bool TWO>
constexpr size_t sk_ffn2_lds_bytes() {
  return SkFfn2Lds<FS, TWO>::kStaged ? SkFfn2Lds<FS, TWO>::kBytes : SkLds<PER>::kBytes;
}

template <int PER, int FS, bool TWO, class WT>   // FS = F / 128 = k steps per wave
__global__ __launch_bounds__(kSkThreads) void sk_ffn2_kernel(SkSrc resid, int R, const bf16* __restrict__ hid,
                                                             const WT* __restrict__ W,
                                                             const float* __restrict__ wscale,
                                                             const bf16* __restrict__ bias,
                                                             float* __restrict__ xs_out) {
  extern __shared__ __attribute__((aligned(16))) char sk_smem[];
  typedef SkFfn2Lds<FS, TWO> FL;
  constexpr int d = 64 * PER, F = 128 * FS, S1 = FS < kSkW ? FS : kSkW;
  const int n0 = blockIdx.x * 16, wave = threadIdx.x >> 6, lq = threadIdx.x & 15, g = (threadIdx.x & 63) >> 4;
  const int k0 = wave * (F / 4);
  const bf16 bias_n = bias[n0 + (threadIdx.x & 15)];   // for the epilogue (sk_reduce: column threadIdx % 16)
  const float ws_n = sk_wscale<WT>(wscale, n0 + (threadIdx.x & 15));
  f32x4 acc[2];
  sk_zero(acc);
  if constexpr (FL::kStaged) {
    bf16* hidl = reinterpret_cast<bf16*>(sk_smem);
    float* hown = reinterpret_cast<float*>(sk_smem + FL::kHid);
    float* red = reinterpret_cast<float*>(sk_smem + FL::kHid + FL::kOwn);
    typename SkFrag<WT>::type wf[S1];
    sk_wload<S1>(W, F, n0, d, k0, wf);
    // one request = 64 lanes x 16 B = 512 columns of a row; wave w takes columns 512 w, 512 (w + 4), ...
    for (int r = 0; r < R; ++r)
      for (int c = wave * 512; c < F; c += 4 * 512)
        __builtin_amdgcn_global_load_lds(SD_GLB_PTR(hid + (size_t)r * F + c + (threadIdx.x & 63) * 8),
                                         SD_LDS_PTR(hidl + r * FL::kPitch + c), 16, 0, 0);
    sk_hidden<PER>(resid, R, TWO ? 32 : 16, nullptr, hown, n0, false);
    __syncthreads();   // (waits for the requests above as well)
    auto getB = [&](int t, int k) {
      return *reinterpret_cast<const bf16x8*>(hidl + (t * 16 + lq) * FL::kPitch + k);
    };
    sk_mma<S1, TWO>(wf, k0, getB, acc);
    sk_mma_tail<FS, TWO>(W, F, n0, d, k0, getB, acc);
    mfma_settle(acc[0], acc[1]);
    __syncthreads();
    sk_reduce(acc, red, R, [&](int m, int nl, float v) {
      xs_out[(size_t)m * d + n0 + nl] = v * ws_n + (float)bias_n + hown[m * 16 + nl];
    });
  } else {
    SkLds<PER> L(sk_smem);
    typename SkFrag<WT>::type wf[S1];
    bf16x8 hf[S1];
    sk_wload<S1>(W, F, n0, d, k0, wf);
    // first-tile activations of the same k range, straight from memory (same operand layout)
    {
      const bf16* hp = hid + (size_t)min(lq, R - 1) * F + k0 + 8 * g;
#pragma unroll
      for (int u = 0; u < S1; ++u) hf[u] = *reinterpret_cast<const bf16x8*>(hp + u * 32);
    }
    sk_hidden<PER>(resid, R, TWO ? 32 : 16, L.hb, L.hown, n0, false);
    auto getB = [&](int t, int k) {
      return *reinterpret_cast<const bf16x8*>(hid + (size_t)min(t * 16 + lq, R - 1) * F + k);
    };
#pragma unroll
    for (int u = 0; u < S1; ++u) {
      const bf16x8 w = sk_frag(wf[u]);
      acc[0] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(w, hf[u], acc[0], 0, 0, 0);
      if (TWO) acc[1] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(w, getB(1, k0 + u * 32 + 8 * g), acc[1], 0, 0, 0);
    }
    sk_mma_tail<FS, TWO>(W, F, n0, d, k0, getB, acc);
    mfma_settle(acc[0], acc[1]);
    __syncthreads();
    const float* hown = L.hown;
    sk_reduce(acc, L.red, R, [&](int m, int nl, float v) {
      xs_out[(size_t)m * d + n0 + nl] = v * ws_n + (float)bias_n + hown[m * 16 + nl];
    });
  }
}

// ------------------------------------------------------------------------------------ vocabulary
// Every block first forms the draft logits itself (waves 0 and 1, the sk_draft_logit sequence on
// its own copy of the hidden rows: the same bits in every block, and the bits its own tile would
// hold for that column), so the rank counts need no launch of their own before this one.
template <int PER, bool TWO, class WT>
__global__ __launch_bounds__(kSkThreads) void sk_vocab_kernel(SkSrc src, int R, const WT* __restrict__ E,
                                                              const float* __restrict__ wscale, int V,
                                                              const int* __restrict__ row_draft,
                                                              float* __restrict__ zd_out,
                                                              float* __restrict__ part, int n_tiles,
                                                              float* __restrict__ logits) {
  extern __shared__ __attribute__((aligned(16))) char sk_smem[];
  SkLds<PER> L(sk_smem);
  constexpr int d = 64 * PER, pitch = d + kSkPad;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, lq = lane & 15;
  const int n0 = blockIdx.x * 64 + wave * 16;
  constexpr int steps = d / 32, S1 = steps < kSkW ? steps : kSkW;
  typename SkFrag<WT>::type wf[S1];
  const int dtok = sk_draft_tok(R, row_draft);   // first: the draft's embedding row then travels with the tile
  sk_wload<S1>(E, d, n0, V, 0, wf);
  SkDraft<PER, WT> dr;
  sk_draft_fetch<PER, WT>(dr, R, E, V, dtok, wscale);
  float ws[4];   // this lane's columns n0 + 4 (lane / 16) + r
#pragma unroll
  for (int r = 0; r < 4; ++r) ws[r] = sk_wscale<WT>(wscale, min(n0 + 4 * (lane >> 4) + r, V - 1));
  sk_hidden<PER>(src, R, TWO ? 32 : 16, L.hb, L.hown, -64, true);
  __syncthreads();
  float* zds = L.hown;   // [32] (the residual slices are not used by this kernel)
  sk_draft_logit<PER, WT>(dr, L.hb, R, [&](int row, float v) {
    zds[row] = v;
    if (blockIdx.x == 0) zd_out[row] = v;
  });
  f32x4 acc[2];
  sk_zero(acc);
  const bf16* hb = L.hb;
  auto getB = [&](int t, int k) { return *reinterpret_cast<const bf16x8*>(hb + (t * 16 + lq) * pitch + k); };
  sk_mma<S1, TWO>(wf, 0, getB, acc);
  sk_mma_tail<steps, TWO>(E, d, n0, V, 0, getB, acc);
  if constexpr (!std::is_same<WT, bf16>::value) {
#pragma unroll
    for (int t = 0; t < 2; ++t)
#pragma unroll
      for (int r = 0; r < 4; ++r) acc[t][r] *= ws[r];
  }
  __syncthreads();
  float zd[2];
#pragma unroll
  for (int t = 0; t < 2; ++t) zd[t] = (t * 16 + lq < R) ? zds[t * 16 + lq] : kNegInf;
  sk_vocab_tile(acc, n0, V, R, zd, L.red, part, n_tiles, blockIdx.x, logits);
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

template <int PER, bool TWO, class WT>
static hipError_t sk_init_rows() {
  hipError_t e;
  if ((e = sk_attr<PER>(sk_qkv_kernel<PER, TWO, WT>)) != hipSuccess) return e;
  if ((e = sk_attr<PER>(sk_attn_o_kernel<PER, false, TWO, WT>)) != hipSuccess) return e;
  if ((e = sk_attr<PER>(sk_attn_o_kernel<PER, true, TWO, WT>)) != hipSuccess) return e;
  if ((e = sk_attr<PER>(sk_attn_o_kernel<PER, true, TWO, WT, true>)) != hipSuccess) return e;
  if ((e = sk_attr<PER>(sk_proj_kernel<PER, TWO, WT>)) != hipSuccess) return e;
  if ((e = hipFuncSetAttribute(reinterpret_cast<const void*>(sk_ffn2_kernel<PER, 2, TWO, WT>),
                               hipFuncAttributeMaxDynamicSharedMemorySize, (int)sk_ffn2_lds_bytes<PER, 2, TWO>())) != hipSuccess) return e;
  if ((e = hipFuncSetAttribute(reinterpret_cast<const void*>(sk_ffn2_kernel<PER, 16, TWO, WT>),
                               hipFuncAttributeMaxDynamicSharedMemorySize, (int)sk_ffn2_lds_bytes<PER, 16, TWO>())) != hipSuccess) return e;
  if ((e = hipFuncSetAttribute(reinterpret_cast<const void*>(sk_ffn2_kernel<PER, 32, TWO, WT>),
                               hipFuncAttributeMaxDynamicSharedMemorySize, (int)sk_ffn2_lds_bytes<PER, 32, TWO>())) != hipSuccess) return e;
  if ((e = sk_attr<PER>(sk_vocab_kernel<PER, TWO, WT>)) != hipSuccess) return e;
  return hipSuccess;
}

hipError_t skinny_init(int d) {
  hipError_t e = hipSuccess;
  SK_DISPATCH(d, {
    if ((e = sk_init_rows<PER, false, bf16>()) != hipSuccess) return e;
    if ((e = sk_init_rows<PER, true, bf16>()) != hipSuccess) return e;
    if ((e = sk_init_rows<PER, false, fp8>()) != hipSuccess) return e;
    if ((e = sk_init_rows<PER, true, fp8>()) != hipSuccess) return e;
  });
  return e;
}

// A weight argument is a SkWeight: bf16 values, or (scale != nullptr) E4M3 codes + row scales.
#define SK_WT(w, CALL)                                                                     \
  if ((w).scale) { typedef fp8 WT; const fp8* Wp = static_cast<const fp8*>((w).p); CALL; } \
  else { typedef bf16 WT; const bf16* Wp = static_cast<const bf16*>((w).p); CALL; }

hipError_t skinny_qkv(hipStream_t st, const SkSrc& src, int R, int d, SkWeight W, const bf16* bias, bf16* q,
                      bf16* kc, bf16* vc, const int* row_b, const int* row_pos, int H, int Lcap) {
  SK_DISPATCH(d, SK_ROWS(R, SK_WT(W, hipLaunchKernelGGL((sk_qkv_kernel<PER, TWO, WT>), dim3(3 * d / 16),
                                                        dim3(kSkThreads), SkLds<PER>::kBytesNoAttn, st, src, R, Wp,
                                                        W.scale, bias, q, kc, vc, row_b, row_pos, H, Lcap))));
  return hipGetLastError();
}
hipError_t skinny_attn_o(hipStream_t st, const SkSrc& resid, int R, int d, const AttnArgs& a, SkWeight W,
                         const bf16* bias, float* xs_out) {
  if (a.k_scale || a.v_scale) {   // FP8 cross-attention keys and values
    if (!a.k_scale || !a.v_scale || !a.v_blocked) return hipErrorInvalidValue;
    SK_DISPATCH(d, SK_ROWS(R, SK_WT(W, hipLaunchKernelGGL((sk_attn_o_kernel<PER, true, TWO, WT, true>), dim3(d / 16),
                                                          dim3(64 * kSkAttnWaves), SkLds<PER>::kBytes, st, resid, R, a,
                                                          Wp, W.scale, bias, xs_out))));
  } else if (a.v_blocked) {
    SK_DISPATCH(d, SK_ROWS(R, SK_WT(W, hipLaunchKernelGGL((sk_attn_o_kernel<PER, true, TWO, WT>), dim3(d / 16),
                                                          dim3(64 * kSkAttnWaves), SkLds<PER>::kBytes, st, resid, R, a,
                                                          Wp, W.scale, bias, xs_out))));
  } else {
    SK_DISPATCH(d, SK_ROWS(R, SK_WT(W, hipLaunchKernelGGL((sk_attn_o_kernel<PER, false, TWO, WT>), dim3(d / 16),
                                                          dim3(64 * kSkAttnWaves), SkLds<PER>::kBytes, st, resid, R, a,
                                                          Wp, W.scale, bias, xs_out))));
  }
  return hipGetLastError();
}
hipError_t skinny_proj(hipStream_t st, const SkSrc& src, int R, int d, SkWeight W, int N, const bf16* bias,
                       bf16* out, bool relu) {
  SK_DISPATCH(d, SK_ROWS(R, SK_WT(W, hipLaunchKernelGGL((sk_proj_kernel<PER, TWO, WT>), dim3((N + 15) / 16),
                                                        dim3(kSkThreads), SkLds<PER>::kBytesNoAttn, st, src, R, Wp,
                                                        W.scale, N, bias, out, relu ? 1 : 0))));
  return hipGetLastError();
}
hipError_t skinny_ffn2(hipStream_t st, const SkSrc& resid, int R, int d, const bf16* hid, int F, SkWeight W,
                       const bf16* bias, float* xs_out) {
  SK_DISPATCH(d, SK_FFN(F, SK_ROWS(R, SK_WT(W, hipLaunchKernelGGL((sk_ffn2_kernel<PER, FS, TWO, WT>), dim3(d / 16),
                                                                  dim3(kSkThreads), (sk_ffn2_lds_bytes<PER, FS, TWO>()),
                                                                  st, resid, R, hid, Wp, W.scale, bias, xs_out)))));
  return hipGetLastError();
}
hipError_t skinny_vocab(hipStream_t st, const SkSrc& src, int R, int d, SkWeight E, int V, const int* row_draft,
                        float* zd_row, float* part, float* logits) {
  const int n_tiles = (V + 63) / 64;
  SK_DISPATCH(d, {
    SK_ROWS(R, SK_WT(E, hipLaunchKernelGGL((sk_vocab_kernel<PER, TWO, WT>), dim3(n_tiles), dim3(kSkThreads),
                                           SkLds<PER>::kBytesNoAttn, st, src, R, Wp, E.scale, V, row_draft, zd_row,
                                           part, n_tiles, logits)));
  });
  return hipGetLastError();
}

}  // namespace sd
