// MFMA GEMM kernels of the decoder / encoder blocks and the fused vocabulary kernel.
#include "gemm_core.h"
#include "kernels.h"
#include <type_traits>

namespace sd {

static thread_local KernelTimer* g_kernel_timer = nullptr;
void set_kernel_timer(KernelTimer* t) { g_kernel_timer = t; }
KernelTimer* kernel_timer() { return g_kernel_timer; }

// Workgroup ids are dealt round-robin to the 8 XCDs (id % 8), each with its own L2.  Tiles are
// numbered n-major (m fastest) and XCD x takes the contiguous run [x*per, (x+1)*per): the
// tiles that run together on one XCD then share a few weight column-panels and the
// activation rows, which stay in that XCD's L2.  Returns false for the padding blocks.
__device__ __forceinline__ bool xcd_tile(int MT, int NT, int& mt, int& nt) {
  const int nb = MT * NT, id = blockIdx.x;
  const int per = (nb + 7) >> 3;
  const int t = (id & 7) * per + (id >> 3);
  if ((id >> 3) >= per || t >= nb) return false;
  nt = t / MT;
  mt = t - nt * MT;
  return true;
}
static inline int xcd_grid(int MT, int NT) { return 8 * ((MT * NT + 7) / 8); }

// fp32 staging tile in LDS, [BM][BN]; rows r and r+4 come from the two lane halves of one
// MFMA register, so bit 5 of the column is flipped for every other group of 4 rows.
template <int BN>
__device__ __forceinline__ int cs_off(int row, int col) {
  return row * BN + (col ^ (((row >> 2) & 1) << 5));
}

// ----------------------------------------------------------------------------- epilogues
// An epilogue handles 8 consecutive columns [n, n+8) of row m (n % 8 == 0, inside the matrix)
// in two steps: fetch() issues every global read the chunk needs (bias, residual, row
// bookkeeping), store() consumes them.  The kernel calls fetch() for all chunks of a thread
// before the first store(), so the reads of a tile cost one memory round trip in total.
struct EpiF32 {
  const bf16* __restrict__ bias;
  const float* resid;   // may alias out
  float* out;
  int ldo;
  struct Pre { bf16x8 b; f32x4 r0, r1; };
  __device__ __forceinline__ Pre fetch(int m, int n) const {
    Pre p;
    p.b = *reinterpret_cast<const bf16x8*>(bias + n);
    const size_t o = (size_t)m * ldo + n;
    if (resid) { p.r0 = *reinterpret_cast<const f32x4*>(resid + o); p.r1 = *reinterpret_cast<const f32x4*>(resid + o + 4); }
    else { p.r0 = f32x4{0.f, 0.f, 0.f, 0.f}; p.r1 = p.r0; }
    return p;
  }
  __device__ __forceinline__ void store(int m, int n, const float (&v)[8], const Pre& p) const {
    f32x4 w0, w1;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      w0[i] = v[i] + (float)p.b[i] + p.r0[i];
      w1[i] = v[4 + i] + (float)p.b[4 + i] + p.r1[i];
    }
    const size_t o = (size_t)m * ldo + n;
    *reinterpret_cast<f32x4*>(out + o) = w0;
    *reinterpret_cast<f32x4*>(out + o + 4) = w1;
  }
};

__device__ __forceinline__ bf16x8 pack_bias(const float (&v)[8], const bf16x8& b, bool relu) {
  bf16x8 o;
#pragma unroll
  for (int i = 0; i < 8; ++i) {
    float t = v[i] + (float)b[i];
    if (relu) t = fmaxf(t, 0.f);
    o[i] = (bf16)t;
  }
  return o;
}

struct EpiBf16 {
  const bf16* __restrict__ bias;
  bf16* __restrict__ out;
  int ldo;
  int relu;
  struct Pre { bf16x8 b; };
  __device__ __forceinline__ Pre fetch(int m, int n) const {
    return Pre{*reinterpret_cast<const bf16x8*>(bias + n)};
  }
  __device__ __forceinline__ void store(int m, int n, const float (&v)[8], const Pre& p) const {
    *reinterpret_cast<bf16x8*>(out + (size_t)m * ldo + n) = pack_bias(v, p.b, relu != 0);
  }
};

// Decoder self-attention projection: columns [0,d) are queries, [d,2d) keys, [2d,3d) values.
// Keys and values go straight into the cache rows of the token they belong to: this is the
// "append" of the KV cache, fused into the projection.  Both caches are [B][H][Lcap][64].
struct EpiQkvAppend {
  const bf16* __restrict__ bias;
  bf16* __restrict__ q;
  bf16* __restrict__ kc;
  bf16* __restrict__ vc;
  const int* __restrict__ row_b;
  const int* __restrict__ row_pos;
  int d, H, Lcap;
  struct Pre { bf16x8 b; int sb, pos; };
  __device__ __forceinline__ Pre fetch(int m, int n) const {
    return Pre{*reinterpret_cast<const bf16x8*>(bias + n), row_b[m], row_pos[m]};
  }
  __device__ __forceinline__ void store(int m, int n, const float (&v)[8], const Pre& p) const {
    const bf16x8 o = pack_bias(v, p.b, false);
    const int part = n / d, c = n - part * d;
    if (part == 0) {
      *reinterpret_cast<bf16x8*>(q + (size_t)m * d + c) = o;
      return;
    }
    if (p.sb < 0) return;
    const int h = c >> 6, e = c & 63;
    bf16* cache = (part == 1) ? kc : vc;
    *reinterpret_cast<bf16x8*>(cache + (((size_t)p.sb * H + h) * Lcap + p.pos) * kHeadDim + e) = o;
  }
};

// Cross-attention keys/values of the encoder memory: row m = b*S + s.
//   xk [B][H][Scap][64]     xv [B][H][Scap/8][64][8] (blocked like the value cache)
// Row m of the source side belongs to sequence b at source position s: m = b * S + s for padded
// rows, or (row_b[m], row_s[m]) for packed rows (row_b < 0: a row no sequence owns).
struct SrcRows {
  const int* __restrict__ row_b;   // null: padded rows
  const int* __restrict__ row_s;
  int S;
  struct At { int b, s; };
  __device__ __forceinline__ At at(int m) const {
    if (row_b) return At{row_b[m], row_s[m]};
    const int b = m / S;
    return At{b, m - b * S};
  }
};

struct EpiCrossKv {
  const bf16* __restrict__ bias;
  bf16* __restrict__ xk;
  bf16* __restrict__ xv;
  int d, H, Scap;
  SrcRows rows;
  struct Pre { bf16x8 b; SrcRows::At at; };
  __device__ __forceinline__ Pre fetch(int m, int n) const {
    return Pre{*reinterpret_cast<const bf16x8*>(bias + n), rows.at(m)};
  }
  __device__ __forceinline__ void store(int m, int n, const float (&v)[8], const Pre& p) const {
    const bf16x8 o = pack_bias(v, p.b, false);
    const int part = n / d, c = n - part * d;
    const int b = p.at.b, s = p.at.s;
    if (b < 0) return;
    const int h = c >> 6, e = c & 63;
    if (part == 0) {
      *reinterpret_cast<bf16x8*>(xk + (((size_t)b * H + h) * Scap + s) * kHeadDim + e) = o;
    } else {
      bf16* dst = xv + ((size_t)b * H + h) * Scap * kHeadDim + vt_off(s, e);
#pragma unroll
      for (int i = 0; i < 8; ++i) dst[i * 8] = o[i];
    }
  }
};

// Encoder self-attention projection, N = 3d, row m = b*S + s: queries -> q [M,d]; keys and
// values of the source go into the same layouts as the cross-attention K/V.
struct EpiEncQkv {
  const bf16* __restrict__ bias;
  bf16* __restrict__ q;
  bf16* __restrict__ xk;
  bf16* __restrict__ xv;
  int d, H, Scap;
  SrcRows rows;
  struct Pre { bf16x8 b; SrcRows::At at; };
  __device__ __forceinline__ Pre fetch(int m, int n) const {
    return Pre{*reinterpret_cast<const bf16x8*>(bias + n), rows.at(m)};
  }
  __device__ __forceinline__ void store(int m, int n, const float (&v)[8], const Pre& p) const {
    const bf16x8 o = pack_bias(v, p.b, false);
    const int part = n / d, c = n - part * d;
    if (part == 0) {
      *reinterpret_cast<bf16x8*>(q + (size_t)m * d + c) = o;
      return;
    }
    const int b = p.at.b, s = p.at.s;
    if (b < 0) return;
    const int h = c >> 6, e = c & 63;
    if (part == 1) {
      *reinterpret_cast<bf16x8*>(xk + (((size_t)b * H + h) * Scap + s) * kHeadDim + e) = o;
    } else {
      bf16* dst = xv + ((size_t)b * H + h) * Scap * kHeadDim + vt_off(s, e);
#pragma unroll
      for (int i = 0; i < 8; ++i) dst[i * 8] = o[i];
    }
  }
};

template <class Cfg, class Epi>
__global__ __launch_bounds__(Cfg::kThreads) void gemm_kernel(const bf16* __restrict__ A, int lda,
                                                             const bf16* __restrict__ W, int ldw,
                                                             int M, int N, int K, int MT, int NT,
                                                             Epi epi, const int* __restrict__ m_real) {
  extern __shared__ __attribute__((aligned(1024))) bf16 smem[];
  static_assert(Cfg::kSmemBytes >= Cfg::kBM * Cfg::kBN * 4, "staging tile must fit in the ring");
  int mt, nt;
  if (!xcd_tile(MT, NT, mt, nt)) return;
  const int m0 = mt * Cfg::kBM, n0 = nt * Cfg::kBN;
  if (m_real) {   // only the leading *m_real rows hold data (same value for the whole grid)
    M = min(M, *m_real);
    if (m0 >= M) return;
  }
  constexpr int CPR = Cfg::kBN / 8;                          // 8-column chunks per row
  constexpr int ITER = Cfg::kBM * CPR / Cfg::kThreads;       // chunks per thread
  static_assert(Cfg::kBM * CPR % Cfg::kThreads == 0, "tile / thread count");
  // what the epilogue reads from memory is requested before the K loop and arrives under it
  typename Epi::Pre pre[ITER];
#pragma unroll
  for (int it = 0; it < ITER; ++it) {
    const int idx = it * Cfg::kThreads + threadIdx.x;
    const int r = idx / CPR, c = (idx - r * CPR) * 8;
    pre[it] = epi.fetch(min(m0 + r, M - 1), min(n0 + c, N - 8));
  }
  GemmAcc<Cfg> acc;
  gemm_mainloop<Cfg>(A, lda, W, ldw, M, N, 0, K / Cfg::GK, m0, n0, smem, acc);
  float* cs = reinterpret_cast<float*>(smem);
  gemm_foreach<Cfg>(acc, 0, 0, [&](int r, int c, float v) { cs[cs_off<Cfg::kBN>(r, c)] = v; });
  __syncthreads();
#pragma unroll
  for (int it = 0; it < ITER; ++it) {
    const int idx = it * Cfg::kThreads + threadIdx.x;
    const int r = idx / CPR, c = (idx - r * CPR) * 8;
    const int m = m0 + r, n = n0 + c;
    if (m < M && n < N) {
      const float* src = cs + cs_off<Cfg::kBN>(r, c);
      f32x4 a = *reinterpret_cast<const f32x4*>(src), b = *reinterpret_cast<const f32x4*>(src + 4);
      const float v[8] = {a[0], a[1], a[2], a[3], b[0], b[1], b[2], b[3]};
      epi.store(m, n, v, pre[it]);
    }
  }
}

typedef GemmCfg<128, 128, 2> CfgWide;      // 64 KB LDS: two blocks per CU
typedef GemmCfg<64, 64, 4> CfgSmall;       // 64 KB LDS; many tiles for narrow outputs
typedef GemmCfg<256, 128, 3, 4, 2> CfgTall;   // 144 KB LDS, eight waves: one block per CU

template <class Cfg, class Epi>
static hipError_t launch_cfg(hipStream_t st, const bf16* A, int lda, const bf16* W, int M, int N, int K,
                             const Epi& epi, const int* m_real) {
  // (initialisation of a function-local static is thread-safe)
  static const hipError_t attr = hipFuncSetAttribute(reinterpret_cast<const void*>(gemm_kernel<Cfg, Epi>),
                                                     hipFuncAttributeMaxDynamicSharedMemorySize, Cfg::kSmemBytes);
  if (attr != hipSuccess) return attr;
  const int MT = (M + Cfg::kBM - 1) / Cfg::kBM, NT = (N + Cfg::kBN - 1) / Cfg::kBN;
  SD_LAUNCH_TIMED((gemm_kernel<Cfg, Epi>), dim3(xcd_grid(MT, NT)), dim3(Cfg::kThreads), Cfg::kSmemBytes, st,
                     A, lda, W, K, M, N, K, MT, NT, epi, m_real);
  return hipGetLastError();
}

template <class Epi>
static hipError_t launch(hipStream_t st, const bf16* A, int lda, const bf16* W, int M, int N, int K,
                         const Epi& epi, const int* m_real = nullptr) {
  if (M <= 0 || N <= 0) return hipSuccess;
  // enough 128x128 tiles to give every CU one?  else take 64x64 tiles
  const long wide_tiles = (long)((M + 127) / 128) * ((N + 127) / 128);
  // (a K of 512 is eight stages: a launch is then mostly its tiles' fixed costs, and the small tiles' are smaller)
  if (wide_tiles >= 200 && K > 512) return launch_cfg<CfgWide>(st, A, lda, W, M, N, K, epi, m_real);
  return launch_cfg<CfgSmall>(st, A, lda, W, M, N, K, epi, m_real);
}

hipError_t gemm_f32(hipStream_t st, const bf16* A, int lda, const bf16* W, int M, int N, int K,
                    const bf16* bias, const float* resid, float* out, int ldo, const int* m_real) {
  return launch(st, A, lda, W, M, N, K, EpiF32{bias, resid, out, ldo}, m_real);
}
hipError_t gemm_bf16(hipStream_t st, const bf16* A, int lda, const bf16* W, int M, int N, int K,
                     const bf16* bias, bf16* out, int ldo, bool relu, const int* m_real) {
  return launch(st, A, lda, W, M, N, K, EpiBf16{bias, out, ldo, relu ? 1 : 0}, m_real);
}
hipError_t gemm_qkv_append(hipStream_t st, const bf16* A, const bf16* W, int M, int d, int K,
                           const bf16* bias, bf16* q_out, bf16* kc, bf16* vc, const int* row_b,
                           const int* row_pos, int H, int Lcap, const int* m_real) {
  return launch(st, A, K, W, M, 3 * d, K, EpiQkvAppend{bias, q_out, kc, vc, row_b, row_pos, d, H, Lcap}, m_real);
}
hipError_t gemm_cross_kv(hipStream_t st, const bf16* A, const bf16* W, int M, int d, int K,
                         const bf16* bias, bf16* xk, bf16* xv, int S, int H, int Scap, const int* row_b,
                         const int* row_s, const int* m_real) {
  return launch(st, A, K, W, M, 2 * d, K, EpiCrossKv{bias, xk, xv, d, H, Scap, SrcRows{row_b, row_s, S}}, m_real);
}

hipError_t gemm_enc_qkv(hipStream_t st, const bf16* A, const bf16* W, int M, int d, int K,
                        const bf16* bias, bf16* q_out, bf16* ek, bf16* ev, int S, int H, int Scap, const int* row_b,
                        const int* row_s, const int* m_real) {
  return launch(st, A, K, W, M, 3 * d, K, EpiEncQkv{bias, q_out, ek, ev, d, H, Scap, SrcRows{row_b, row_s, S}}, m_real);
}

// ----------------------------------------------------------------------------- LayerNorm folded into the GEMMs
// Post-LN blocks: x' = LN(y), y = x + sublayer(x).  Instead of a pass of its own over y, the
// normalisation is split between the GEMM that produces y and the GEMMs that consume x':
//   producer (EpiLnSum)   writes y (fp32), bf16(y * g) and, for every 64-column chunk of every row,
//                         the pair {sum, sum of squared deviations from the chunk mean};
//   consumer (EpiLn*)     multiplies bf16(y * g) by the unchanged weights and finishes
//                         LN(y) W^T + b = rstd * (acc - mean * cs) + bf,
//                         cs[n] = sum_k g[k] W[n][k],  bf[n] = b[n] + sum_k beta[k] W[n][k]
//                         (both fp32, derived once per model by ln_fold);
//   the residual x' that the next producer adds is recomputed there from y, mean, rstd, g, beta.
// mean and rstd of a row come from its chunk pairs, merged with the parallel-variance formula;
// eps = 1e-5 and the biased variance, as in layer_norm.  Epilogues run with every wave of the
// chip at the same point and nothing to overlap with, so they are written for few instructions:
// per row {rstd, -mean * rstd}, per column folded constants, fused multiply-adds.
typedef float f32x2 __attribute__((ext_vector_type(2)));

// Sums over aligned groups of 2, 4 or 8 neighbouring lanes with DPP moves (no LDS round trip).
template <int LANES>
__device__ __forceinline__ float group_sum(float v) {
  static_assert(LANES == 2 || LANES == 4 || LANES == 8, "group size");
  v += dpp_f<kDppSwap1>(v);
  if (LANES >= 4) v += dpp_f<kDppSwap2>(v);
  if (LANES >= 8) v += dpp_f<kDppHalfMirror>(v);
  return v;
}

// Chunk pairs of a row lie together, [M][pitch] pairs with pitch = chunks rounded up to even, so a
// thread fetches two pairs per 16-byte load.
__host__ __device__ __forceinline__ int ln_pitch(int chunks) { return (chunks + 1) & ~1; }

template <class Cfg>
struct LnRows {
  static constexpr int TPR = Cfg::kThreads / Cfg::kBM;   // threads that share one tile row
  static constexpr int NL = 16 / TPR;                    // 16-byte loads per thread (d <= 2048)
  static_assert(TPR == 2 || TPR == 4, "threads per row");
  f32x4 p[NL];                                           // pairs 2q, 2q+1 for q = j + i * TPR
  // Loads sit behind conditions on kernel arguments only (no lane takes a branch of its own).
  __device__ __forceinline__ void request(const f32x2* part, int chunks, int m0, int M) {
    const int r = threadIdx.x / TPR, j = threadIdx.x % TPR;
    const int pitch = ln_pitch(chunks);
    const f32x4* src = reinterpret_cast<const f32x4*>(part + (size_t)min(m0 + r, M - 1) * pitch);
#pragma unroll
    for (int i = 0; i < NL; ++i) {
      p[i] = f32x4{0.f, 0.f, 0.f, 0.f};
      if (2 * i * TPR < chunks) p[i] = src[min(j + i * TPR, pitch / 2 - 1)];
    }
  }
  // rowstat [BM][2] in LDS: {rstd, -mean * rstd}; {1, 0} when there is nothing to normalise
  __device__ __forceinline__ void finish(int chunks, bool identity, float* rowstat) const {
    const int r = threadIdx.x / TPR, j = threadIdx.x % TPR;
    const float inv_d = __builtin_amdgcn_rcpf((float)(64 * chunks));   // d = 2^6 * chunks: exact for powers of two
    float s = 0.f;
#pragma unroll
    for (int i = 0; i < NL; ++i) {
      if (2 * i * TPR >= chunks) continue;
      const int c = 2 * (j + i * TPR);
      s += (c < chunks ? p[i][0] : 0.f) + (c + 1 < chunks ? p[i][2] : 0.f);
    }
    s = group_sum<TPR>(s);
    const float mean = s * inv_d;
    float q = 0.f;
#pragma unroll
    for (int i = 0; i < NL; ++i) {
      if (2 * i * TPR >= chunks) continue;
      const int c = 2 * (j + i * TPR);
      const float d0 = p[i][0] * (1.0f / 64.0f) - mean, d1 = p[i][2] * (1.0f / 64.0f) - mean;
      q += (c < chunks ? p[i][1] + 64.0f * d0 * d0 : 0.f) + (c + 1 < chunks ? p[i][3] + 64.0f * d1 * d1 : 0.f);
    }
    q = group_sum<TPR>(q);
    if (j == 0) {
      const float rstd = identity ? 1.f : fast_rsqrt(q * inv_d + 1e-5f);
      rowstat[2 * r] = rstd;
      rowstat[2 * r + 1] = identity ? 0.f : -mean * rstd;
    }
  }
};

// Producer.  x holds the previous sum y_prev (or the plain residual when has_prev is 0) and
// receives the new sum in place.  Column vectors (LnSumVecs, fp32 [3][d]):
//   0: gain of the LayerNorm pending on x (1 without one)
//   1: its shift (0 without one) + this GEMM's bias
//   2: gain of the LayerNorm that follows
struct EpiLnSum {
  static constexpr int kVec = 3;
  const float* __restrict__ vecs;
  const f32x2* ln_in;              // chunk pairs of y_prev
  f32x2* ln_out;                   // chunk pairs of the new sum
  float* x;
  bf16* __restrict__ xg;           // bf16(y * next gain)
  int ld, chunks;
  int has_prev;                    // 0: x is the residual itself
  __device__ __forceinline__ const float* vec(int i) const { return vecs + i * ld; }
  __device__ __forceinline__ bool identity() const { return has_prev == 0; }
  struct Pre { f32x4 r0, r1; };
  __device__ __forceinline__ Pre fetch(int m, int n) const {
    const size_t o = (size_t)m * ld + n;
    return Pre{*reinterpret_cast<const f32x4*>(x + o), *reinterpret_cast<const f32x4*>(x + o + 4)};
  }
  // called by every lane (live = inside the matrix): the chunk sums cross lanes
  __device__ __forceinline__ void store(int m, int n, bool live, const float (&v)[8], const Pre& p,
                                        float rstd, float nmr, const float (&cv)[kVec][8]) const {
    float y[8], s = 0.f, ss = 0.f;
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      const float r = i < 4 ? p.r0[i] : p.r1[i - 4];
      y[i] = v[i] + __builtin_fmaf(__builtin_fmaf(r, rstd, nmr), cv[0][i], cv[1][i]);
      s += y[i];
      ss = __builtin_fmaf(y[i], y[i], ss);
    }
    s = group_sum<8>(s);     // 8 lanes = one 64-column chunk
    ss = group_sum<8>(ss);
    if (!live) return;
    const size_t o = (size_t)m * ld + n;
    *reinterpret_cast<f32x4*>(x + o) = f32x4{y[0], y[1], y[2], y[3]};
    *reinterpret_cast<f32x4*>(x + o + 4) = f32x4{y[4], y[5], y[6], y[7]};
    bf16x8 g;
#pragma unroll
    for (int i = 0; i < 8; ++i) g[i] = (bf16)(y[i] * cv[2][i]);
    *reinterpret_cast<bf16x8*>(xg + o) = g;
    // squared deviations from the chunk mean = sum y^2 - (sum y)^2 / 64, never below 0
    if ((n & 63) == 0) ln_out[(size_t)m * ln_pitch(chunks) + (n >> 6)] = f32x2{s, fmaxf(ss - s * s * (1.0f / 64.0f), 0.f)};
  }
};

// rstd * (acc - mean * cs) + bf on 8 columns: cv[0] = cs, cv[1] = bf
__device__ __forceinline__ bf16x8 ln_finish(const float (&v)[8], float rstd, float nmr, const float (&cv)[2][8],
                                            bool relu) {
  bf16x8 o;
#pragma unroll
  for (int i = 0; i < 8; ++i) {
    float t = __builtin_fmaf(v[i], rstd, __builtin_fmaf(nmr, cv[0][i], cv[1][i]));
    if (relu) t = fmaxf(t, 0.f);
    o[i] = (bf16)t;
  }
  return o;
}

struct EpiLnBf16 {
  static constexpr int kVec = 2;
  const float* __restrict__ cs;
  const float* __restrict__ bf;
  const f32x2* ln_in;
  bf16* __restrict__ out;
  int ldo, chunks, relu;
  __device__ __forceinline__ const float* vec(int i) const { return i == 0 ? cs : bf; }
  __device__ __forceinline__ bool identity() const { return false; }
  struct Pre {};
  __device__ __forceinline__ Pre fetch(int, int) const { return Pre{}; }
  __device__ __forceinline__ void store(int m, int n, bool live, const float (&v)[8], const Pre&,
                                        float rstd, float nmr, const float (&cv)[kVec][8]) const {
    if (live) *reinterpret_cast<bf16x8*>(out + (size_t)m * ldo + n) = ln_finish(v, rstd, nmr, cv, relu != 0);
  }
};

struct EpiLnQkvAppend {
  static constexpr int kVec = 2;
  const float* __restrict__ cs;
  const float* __restrict__ bf;
  const f32x2* ln_in;
  int chunks;
  bf16* __restrict__ q;
  bf16* __restrict__ kc;
  bf16* __restrict__ vc;
  const int* __restrict__ row_b;
  const int* __restrict__ row_pos;
  int d, H, Lcap;
  __device__ __forceinline__ const float* vec(int i) const { return i == 0 ? cs : bf; }
  __device__ __forceinline__ bool identity() const { return false; }
  struct Pre { int sb, pos; };
  __device__ __forceinline__ Pre fetch(int m, int) const { return Pre{row_b[m], row_pos[m]}; }
  __device__ __forceinline__ void store(int m, int n, bool live, const float (&v)[8], const Pre& p,
                                        float rstd, float nmr, const float (&cv)[kVec][8]) const {
    if (!live) return;
    const bf16x8 o = ln_finish(v, rstd, nmr, cv, false);
    const int part = n / d, cc = n - part * d;
    if (part == 0) {
      *reinterpret_cast<bf16x8*>(q + (size_t)m * d + cc) = o;
      return;
    }
    if (p.sb < 0) return;
    const int h = cc >> 6, e = cc & 63;
    bf16* cache = (part == 1) ? kc : vc;
    *reinterpret_cast<bf16x8*>(cache + (((size_t)p.sb * H + h) * Lcap + p.pos) * kHeadDim + e) = o;
  }
};

template <class Cfg, int VEC>
constexpr int ln_smem_bytes() { return Cfg::kSmemBytes + (2 * Cfg::kBM + VEC * Cfg::kBN) * 4; }

template <class Cfg, class Epi>
__global__ __launch_bounds__(Cfg::kThreads) void gemm_ln_kernel(const bf16* __restrict__ A, int lda,
                                                                const bf16* __restrict__ W, int ldw,
                                                                int M, int N, int K, int MT, int NT,
                                                                Epi epi, const int* __restrict__ m_real) {
  extern __shared__ __attribute__((aligned(1024))) bf16 smem[];
  static_assert(Cfg::kSmemBytes >= Cfg::kBM * Cfg::kBN * 4, "staging tile must fit in the ring");
  static_assert(Cfg::kThreads >= Epi::kVec * Cfg::kBN / 4, "one thread per 4 entries of the column vectors");
  float* rowstat = reinterpret_cast<float*>(reinterpret_cast<char*>(smem) + Cfg::kSmemBytes);   // [BM][2]
  float* colv = rowstat + 2 * Cfg::kBM;                                                          // [kVec][BN]
  int mt, nt;
  if (!xcd_tile(MT, NT, mt, nt)) return;
  const int m0 = mt * Cfg::kBM, n0 = nt * Cfg::kBN;
  if (m_real) {   // only the leading *m_real rows hold data (same value for the whole grid)
    M = min(M, *m_real);
    if (m0 >= M) return;
  }
  constexpr int CPR = Cfg::kBN / 8;                    // 8-column pieces per tile row
  constexpr int RPI = Cfg::kThreads / CPR;             // tile rows covered by one pass of the block
  constexpr int ITER = Cfg::kBM / RPI;
  static_assert(Cfg::kThreads % CPR == 0 && Cfg::kBM % RPI == 0, "tile / thread count");
  // a thread keeps its 8 columns in every pass: what depends on the column alone is computed once
  const int tr = threadIdx.x / CPR, tc = (threadIdx.x % CPR) * 8;
  const int n = n0 + tc;
  // everything the epilogue reads is requested here and arrives under the K loop
  LnRows<Cfg> rows;
  rows.request(epi.ln_in, epi.chunks, m0, M);
  constexpr int QPV = Cfg::kBN / 4;   // 16-byte pieces per column vector of the tile
  const bool vec_thread = threadIdx.x < Epi::kVec * QPV;
  f32x4 cvec = {0.f, 0.f, 0.f, 0.f};
  if (vec_thread) cvec = *reinterpret_cast<const f32x4*>(epi.vec(threadIdx.x / QPV) + min(n0 + (int)(threadIdx.x % QPV) * 4, N - 4));
  typename Epi::Pre pre[ITER];
#pragma unroll
  for (int it = 0; it < ITER; ++it) pre[it] = epi.fetch(min(m0 + it * RPI + tr, M - 1), min(n, N - 8));
  GemmAcc<Cfg> acc;
  gemm_mainloop<Cfg>(A, lda, W, ldw, M, N, 0, K / Cfg::GK, m0, n0, smem, acc);
  float* cs = reinterpret_cast<float*>(smem);
  gemm_foreach<Cfg>(acc, 0, 0, [&](int r, int c, float v) { cs[cs_off<Cfg::kBN>(r, c)] = v; });
  rows.finish(epi.chunks, epi.identity(), rowstat);
  if (vec_thread) *reinterpret_cast<f32x4*>(colv + threadIdx.x * 4) = cvec;
  __syncthreads();
  float cv[Epi::kVec][8];
#pragma unroll
  for (int i = 0; i < Epi::kVec; ++i) {
    const f32x4 a = *reinterpret_cast<const f32x4*>(colv + i * Cfg::kBN + tc);
    const f32x4 b = *reinterpret_cast<const f32x4*>(colv + i * Cfg::kBN + tc + 4);
#pragma unroll
    for (int e = 0; e < 4; ++e) { cv[i][e] = a[e]; cv[i][4 + e] = b[e]; }
  }
#pragma unroll
  for (int it = 0; it < ITER; ++it) {
    const int r = it * RPI + tr, m = m0 + r;
    const float* src = cs + cs_off<Cfg::kBN>(r, tc);
    const f32x4 a = *reinterpret_cast<const f32x4*>(src), b = *reinterpret_cast<const f32x4*>(src + 4);
    const f32x2 st = *reinterpret_cast<const f32x2*>(rowstat + 2 * r);
    const float v[8] = {a[0], a[1], a[2], a[3], b[0], b[1], b[2], b[3]};
    epi.store(m, n, m < M && n < N, v, pre[it], st[0], st[1], cv);
  }
}

template <class Cfg, class Epi>
static hipError_t launch_ln_cfg(hipStream_t st, const bf16* A, int lda, const bf16* W, int M, int N, int K,
                                const Epi& epi, const int* m_real) {
  constexpr int kBytes = ln_smem_bytes<Cfg, Epi::kVec>();
  static const hipError_t attr = hipFuncSetAttribute(reinterpret_cast<const void*>(gemm_ln_kernel<Cfg, Epi>),
                                                     hipFuncAttributeMaxDynamicSharedMemorySize, kBytes);
  if (attr != hipSuccess) return attr;
  const int MT = (M + Cfg::kBM - 1) / Cfg::kBM, NT = (N + Cfg::kBN - 1) / Cfg::kBN;
  SD_LAUNCH_TIMED((gemm_ln_kernel<Cfg, Epi>), dim3(xcd_grid(MT, NT)), dim3(Cfg::kThreads), kBytes, st,
                     A, lda, W, K, M, N, K, MT, NT, epi, m_real);
  return hipGetLastError();
}
template <class Epi>
static hipError_t launch_ln(hipStream_t st, const bf16* A, int lda, const bf16* W, int M, int N, int K,
                            const Epi& epi, const int* m_real) {
  if (M <= 0 || N <= 0) return hipSuccess;
  const long wide_tiles = (long)((M + 127) / 128) * ((N + 127) / 128);
  // the widest outputs (QKV and FFN1 of the big model) run on 256x128 tiles, eight waves, three-deep
  // ring: 9-15 % faster than 128x128 on weights streamed from HBM, a few % inside the decoder pass
  if constexpr (Epi::kVec == 2) {
    if (N >= 3072 && M >= 1024) return launch_ln_cfg<CfgTall>(st, A, lda, W, M, N, K, epi, m_real);
  }
  if (wide_tiles >= 200 && K > 512) return launch_ln_cfg<CfgWide>(st, A, lda, W, M, N, K, epi, m_real);
  return launch_ln_cfg<CfgSmall>(st, A, lda, W, M, N, K, epi, m_real);
}

hipError_t gemm_ln_sum(hipStream_t st, const bf16* A, int lda, const bf16* W, int M, int d, int K,
                       const float* vecs, const float* ln_in, bool has_prev, float* x, bf16* xg, float* ln_out,
                       const int* m_real) {
  return launch_ln(st, A, lda, W, M, d, K,
                   EpiLnSum{vecs, reinterpret_cast<const f32x2*>(ln_in), reinterpret_cast<f32x2*>(ln_out), x, xg, d,
                            d / 64, has_prev ? 1 : 0}, m_real);
}
hipError_t gemm_ln_bf16(hipStream_t st, const bf16* A, const bf16* W, int M, int N, int d, const LnFold& f,
                        const float* ln_in, bf16* out, int ldo, bool relu, const int* m_real) {
  return launch_ln(st, A, d, W, M, N, d,
                   EpiLnBf16{f.cs, f.bf, reinterpret_cast<const f32x2*>(ln_in), out, ldo, d / 64, relu ? 1 : 0}, m_real);
}
hipError_t gemm_ln_qkv_append(hipStream_t st, const bf16* A, const bf16* W, int M, int d, const LnFold& f,
                              const float* ln_in, bf16* q_out, bf16* kc, bf16* vc, const int* row_b,
                              const int* row_pos, int H, int Lcap, const int* m_real) {
  return launch_ln(st, A, d, W, M, 3 * d, d,
                   EpiLnQkvAppend{f.cs, f.bf, reinterpret_cast<const f32x2*>(ln_in), d / 64, q_out, kc, vc, row_b,
                                  row_pos, d, H, Lcap}, m_real);
}

// cs[n] = sum_k g[k] W[n][k],  bf[n] = b[n] + sum_k beta[k] W[n][k]; one wave per column n
__global__ __launch_bounds__(256) void ln_fold_kernel(const bf16* __restrict__ W, const bf16* __restrict__ g,
                                                      const bf16* __restrict__ beta, const bf16* __restrict__ b,
                                                      int N, int K, float* __restrict__ cs, float* __restrict__ bf) {
  const int n = blockIdx.x * 4 + (threadIdx.x >> 6), lane = threadIdx.x & 63;
  if (n >= N) return;
  const bf16* w = W + (size_t)n * K;
  float s = 0.f, t = 0.f;
  for (int k = lane; k < K; k += 64) {
    const float wk = (float)w[k];
    s += (float)g[k] * wk;
    t += (float)beta[k] * wk;
  }
  s = wave_sum(s);
  t = wave_sum(t);
  if (lane == 0) { cs[n] = s; bf[n] = (float)b[n] + t; }
}
hipError_t ln_fold(hipStream_t st, const bf16* W, const bf16* g, const bf16* beta, const bf16* b, int N, int K,
                   const LnFold& out) {
  hipLaunchKernelGGL(ln_fold_kernel, dim3((N + 3) / 4), dim3(256), 0, st, W, g, beta, b, N, K,
                     const_cast<float*>(out.cs), const_cast<float*>(out.bf));
  return hipGetLastError();
}

__global__ void ln_sum_vecs_kernel(const bf16* __restrict__ bias, const bf16* __restrict__ gp,
                                   const bf16* __restrict__ bp, const bf16* __restrict__ gn, int d,
                                   float* __restrict__ out) {
  const int n = blockIdx.x * blockDim.x + threadIdx.x;
  if (n >= d) return;
  out[n] = gp ? (float)gp[n] : 1.f;
  out[d + n] = (float)bias[n] + (bp ? (float)bp[n] : 0.f);
  out[2 * d + n] = (float)gn[n];
}
hipError_t ln_sum_vecs(hipStream_t st, const bf16* bias, const bf16* g_prev, const bf16* b_prev, const bf16* g_next,
                       int d, float* out) {
  hipLaunchKernelGGL(ln_sum_vecs_kernel, dim3((d + 255) / 256), dim3(256), 0, st, bias, g_prev, b_prev, g_next, d, out);
  return hipGetLastError();
}

// ----------------------------------------------------------------------------- vocabulary
// Rank test without a sort (paper Eq. 8): the draft is inside the top beta iff fewer than
// beta logits are strictly larger than its own.  Its logit z_d is needed before the big
// product is scanned, so a tiny pre-pass computes it -- with the SAME instruction sequence
// (MFMA 32x32x16, k blocks of 16 in ascending order, same operand roles) that produces that
// very element in the main kernel.  The two values are therefore bit-identical and the
// count is exactly the count over the row the main kernel sees.
//
// One wave = 32 rows: D[i][j] = x_i . E[draft_j]; the diagonal is kept.
template <bool SWAP>
__global__ __launch_bounds__(64) void draft_logit_kernel(const bf16* __restrict__ A, const bf16* __restrict__ E,
                                                         int M, int V, int K, const int* __restrict__ row_draft,
                                                         float* __restrict__ zd_out) {
  const int lane = threadIdx.x, lrow = lane & 31, lhalf = lane >> 5;
  const int r = blockIdx.x * 32 + lrow;
  const int rr = min(r, M - 1);
  const int t = row_draft[rr];
  const bool has = (r < M) && t >= 0 && t < V;
  const bf16* ap = A + (size_t)rr * K + lhalf * 8;
  const bf16* bp = E + (size_t)(has ? t : 0) * K + lhalf * 8;
  f32x16 acc;
#pragma unroll
  for (int i = 0; i < 16; ++i) acc[i] = 0.f;
  // operands of 16 k-blocks are requested together (one memory round trip per 256 columns of K
  // instead of one per block); the accumulation order stays k-ascending
  constexpr int U = 16;
  const int nkb = K / 16;
  for (int kb0 = 0; kb0 < nkb; kb0 += U) {
    bf16x8 a[U], b[U];
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const int kb = min(kb0 + u, nkb - 1);
      a[u] = *reinterpret_cast<const bf16x8*>(ap + kb * 16);
      b[u] = *reinterpret_cast<const bf16x8*>(bp + kb * 16);
    }
    if (kb0 + U <= nkb) {
#pragma unroll
      for (int u = 0; u < U; ++u)
        acc = SWAP ? __builtin_amdgcn_mfma_f32_32x32x16_bf16(b[u], a[u], acc, 0, 0, 0)
                   : __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[u], b[u], acc, 0, 0, 0);
    } else {
      for (int u = 0; u < nkb - kb0; ++u) {
        bf16x8 au = a[0], bu = b[0];
#pragma unroll
        for (int v = 1; v < U; ++v) if (v == u) { au = a[v]; bu = b[v]; }
        acc = SWAP ? __builtin_amdgcn_mfma_f32_32x32x16_bf16(bu, au, acc, 0, 0, 0)
                   : __builtin_amdgcn_mfma_f32_32x32x16_bf16(au, bu, acc, 0, 0, 0);
      }
    }
  }
  mfma_settle(acc);
  // element (i, j): j = lane%32, i = 8*(reg/4) + 4*(lane/32) + reg%4; the diagonal j = i sits in
  // the lane half (j/4)%2, register 4*(j/8) + j%4
  if (lhalf == ((lrow >> 2) & 1) && r < M) {
    const int reg = 4 * (lrow >> 3) + (lrow & 3);
    float v = 0.f;
#pragma unroll
    for (int i = 0; i < 16; ++i) if (i == reg) v = acc[i];
    zd_out[r] = has ? v : kNegInf;
  }
}

// One block = 128 rows x 128 vocabulary columns.  After the K loop the fp32 tile goes through
// LDS so that two threads own one row (64 columns each); each scans its columns once for
// max / arg-max / number of logits above the draft's and once for the sum of exponentials, the
// two halves are merged with lane shuffles, and one 16-byte partial record per (row, tile) is
// written.  Logits never reach memory unless the caller asks for them.
typedef GemmCfg<128, 128, 2> CfgVocab;

// Staging tile of the vocabulary kernel: [128 rows][32 chunks of 4 columns], chunk ch of row r
// at chunk (ch & 16) + ((ch & 15) ^ (r & 15) ^ ((ch >> 4) << 3)): the 16 lanes that read one
// 16-byte chunk each in the same cycle (8 rows x 2 halves) then cover all 64 banks.
__device__ __forceinline__ int vs_off(int row, int ch) {
  return row * 128 + (((ch & 16) + ((ch & 15) ^ (row & 15) ^ ((ch >> 4) << 3))) << 2);
}

// ARGMAX: rows that score no draft and whose log-sum-exp nobody reads (the drafter's slots):
// only max / arg-max are formed; the record's sum is 0 and its count 0.
template <bool ARGMAX>
__global__ __launch_bounds__(CfgVocab::kThreads) void vocab_kernel(const bf16* __restrict__ A,
                                                                   const bf16* __restrict__ E, int M,
                                                                   int V, int K, int MT, int NT,
                                                                   const float* __restrict__ zd_row,
                                                                   float* __restrict__ part,
                                                                   float* __restrict__ logits) {
  extern __shared__ __attribute__((aligned(1024))) bf16 smem[];
  int mt, nt;
  if (!xcd_tile(MT, NT, mt, nt)) return;
  const int m0 = mt * 128, n0 = nt * 128;
  GemmAcc<CfgVocab> acc;
  gemm_mainloop<CfgVocab>(A, K, E, K, M, V, 0, K / CfgVocab::GK, m0, n0, smem, acc);
  float* cs = reinterpret_cast<float*>(smem);  // [128][128] fp32 = 64 KB
  gemm_foreach<CfgVocab>(acc, 0, 0, [&](int r, int c, float v) { cs[vs_off(r, c >> 2) + (c & 3)] = v; });
  __syncthreads();

  const int tid = threadIdx.x;
  const int row = tid >> 1, half = tid & 1;
  const int m = m0 + row;
  const float zd = (zd_row && m < M) ? zd_row[m] : kNegInf;   // -inf on rows that score no draft: count unused
  float best = kNegInf;
  int besti = 0x7fffffff, cnt = 0;
  const bool full = n0 + 128 <= V;
  // thread (row, half) owns columns [half*64, half*64 + 64) of its row: 16 reads of 4 columns
  f32x4 vals[16];
#pragma unroll
  for (int i = 0; i < 16; ++i) vals[i] = *reinterpret_cast<const f32x4*>(cs + vs_off(row, half * 16 + i));
#pragma unroll
  for (int i = 0; i < 16; ++i)
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      const int n = n0 + half * 64 + i * 4 + e;   // ascending: ">" keeps the lowest index of a tie
      const float v = vals[i][e];
      if (full || n < V) {
        if (v > best) { best = v; besti = n; }
        if (!ARGMAX) cnt += (v > zd) ? 1 : 0;
      }
    }
  float se = 0.f;
  if (!ARGMAX) {
#pragma unroll
    for (int i = 0; i < 16; ++i)
#pragma unroll
      for (int e = 0; e < 4; ++e)
        if (full || n0 + half * 64 + i * 4 + e < V) se += __expf(vals[i][e] - best);
  }
  // merge the two halves of the row (lanes tid and tid^1)
  const float obest = __shfl_xor(best, 1, 64);
  const int obesti = __shfl_xor(besti, 1, 64);
  const float ose = __shfl_xor(se, 1, 64);
  const int ocnt = __shfl_xor(cnt, 1, 64);
  const float nb = fmaxf(best, obest);
  float tot = 0.f;
  if (best > kNegInf) tot += se * __expf(best - nb);
  if (obest > kNegInf) tot += ose * __expf(obest - nb);
  const int nbi = (obest > best || (obest == best && obesti < besti)) ? obesti : besti;
  if (half == 0 && m < M) {
    f32x4 rec = {nb, __int_as_float(nbi), tot, __int_as_float(cnt + ocnt)};
    *reinterpret_cast<f32x4*>(part + ((size_t)m * NT + nt) * kPartF) = rec;
  }
  if (logits) {
    for (int idx = tid; idx < 128 * 128; idx += CfgVocab::kThreads) {
      int r = idx >> 7, c = idx & 127;
      if (m0 + r < M && n0 + c < V) logits[(size_t)(m0 + r) * V + n0 + c] = cs[vs_off(r, c >> 2) + (c & 3)];
    }
  }
}

// Many rows (the batched verify and draft passes): one block = 256 rows x 256 vocabulary columns,
// 8 waves (2 along rows x 4 along the vocabulary), which halves what the operand tiles pull through
// L2 per output.  The product is formed transposed (gemm_mainloop<.., SWAP>): a lane then owns 32
// columns of each of its 4 rows, so a row's statistics are a serial scan of the lane's own
// accumulators -- no staging of the fp32 tile through LDS -- followed by one exchange between the lane
// halves and a merge of the two waves that share a 128-column tile through 16 KB of LDS.  The
// partial records keep the 128-column granularity of the kernel above.
typedef GemmCfg<256, 256, 2, 2, 4> CfgVocab256;

template <bool ARGMAX>
__global__ __launch_bounds__(CfgVocab256::kThreads) void vocab256_kernel(const bf16* __restrict__ A,
                                                                         const bf16* __restrict__ E, int M, int V,
                                                                         int K, int MT, int NT256, int NT,
                                                                         const float* __restrict__ zd_row,
                                                                         float* __restrict__ part,
                                                                         float* __restrict__ logits) {
  extern __shared__ __attribute__((aligned(1024))) bf16 smem[];
  int mt, nt;
  if (!xcd_tile(MT, NT256, mt, nt)) return;
  const int m0 = mt * 256, n0 = nt * 256;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wy = wave >> 2, wx = wave & 3, lcol = lane & 31, lhalf = lane >> 5;
  float zd[4];
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const int m = m0 + wy * 128 + i * 32 + lcol;
    zd[i] = (zd_row && m < M) ? zd_row[m] : kNegInf;   // -inf on rows that score no draft: count unused
  }
  GemmAcc<CfgVocab256> acc;
  gemm_mainloop<CfgVocab256, true>(A, K, E, K, M, V, 0, K / CfgVocab256::GK, m0, n0, smem, acc);
  f32x4* rec = reinterpret_cast<f32x4*>(smem);   // [4 wave columns][256 rows]; the ring is free after the main loop
  const int nw = n0 + wx * 64 + 4 * lhalf;        // first column of this lane
  // column of accumulator (j, r) relative to nw: ascending in (j, r), so ">" keeps the lowest index of a tie
  auto col = [](int j, int r) { return j * 32 + 8 * (r >> 2) + (r & 3); };
  constexpr float kLog2e = 1.44269504088896341f;
  auto scan = [&](auto full_tag) {
    constexpr bool FULL = decltype(full_tag)::value;
    const int nvalid = V - nw;   // columns of this lane inside the matrix (FULL: all of them)
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      float best = kNegInf;
      int bestc = 0x3fffffff, cnt = 0;
#pragma unroll
      for (int j = 0; j < 2; ++j)
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          const float v = acc.c[i][j][r];
          if (FULL || col(j, r) < nvalid) {
            if (v > best) { best = v; bestc = col(j, r); }
            if (!ARGMAX) cnt += (v > zd[i]) ? 1 : 0;
          }
        }
      float se = 0.f;
      if (!ARGMAX) {
        const float nb2 = -best * kLog2e;   // exp(v - best) = 2^(v log2e - best log2e)
#pragma unroll
        for (int j = 0; j < 2; ++j)
#pragma unroll
          for (int r = 0; r < 16; ++r)
            if (FULL || col(j, r) < nvalid) se += __builtin_amdgcn_exp2f(__builtin_fmaf(acc.c[i][j][r], kLog2e, nb2));
        if (!(best > kNegInf)) se = 0.f;    // no valid column (or all -inf): nothing to sum
      }
      const int besti = nw + bestc;
      // the other lane half holds the interleaved groups of 4 columns of the same row
      const float obest = __shfl_xor(best, 32, 64);
      const int obesti = __shfl_xor(besti, 32, 64);
      const float ose = __shfl_xor(se, 32, 64);
      const int ocnt = __shfl_xor(cnt, 32, 64);
      const float nb = fmaxf(best, obest);
      float tot = 0.f;
      if (best > kNegInf) tot += se * __expf(best - nb);
      if (obest > kNegInf) tot += ose * __expf(obest - nb);
      const int nbi = (obest > best || (obest == best && obesti < besti)) ? obesti : besti;
      if (lhalf == 0)
        rec[wx * 256 + wy * 128 + i * 32 + lcol] = f32x4{nb, __int_as_float(nbi), tot, __int_as_float(cnt + ocnt)};
    }
  };
  if (n0 + 256 <= V) scan(std::true_type{});
  else scan(std::false_type{});
  if (logits) {
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int m = m0 + wy * 128 + i * 32 + lcol;
#pragma unroll
      for (int j = 0; j < 2; ++j)
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          const int n = nw + j * 32 + 8 * (r >> 2) + (r & 3);
          if (m < M && n < V) logits[(size_t)m * V + n] = acc.c[i][j][r];
        }
    }
  }
  __syncthreads();
  // thread (row, 128-column tile): waves 2t and 2t+1 of the row, lower columns first
  const int row = tid & 255, ct = tid >> 8;
  const int m = m0 + row, nt128 = nt * 2 + ct;
  if (m < M && nt128 < NT) {
    const f32x4 a = rec[(2 * ct) * 256 + row], b = rec[(2 * ct + 1) * 256 + row];
    const float nb = fmaxf(a[0], b[0]);
    float tot = 0.f;
    if (a[0] > kNegInf) tot += a[2] * __expf(a[0] - nb);
    if (b[0] > kNegInf) tot += b[2] * __expf(b[0] - nb);
    const bool tb = b[0] > a[0];   // equal maxima: the lower columns (a) win
    f32x4 out = {nb, tb ? b[1] : a[1], tot, __int_as_float(__float_as_int(a[3]) + __float_as_int(b[3]))};
    *reinterpret_cast<f32x4*>(part + ((size_t)m * NT + nt128) * kPartF) = out;
  }
}

int vocab_tile_cols(int) { return CfgVocab::kBN; }

hipError_t vocab_stats(hipStream_t st, const bf16* A, const bf16* E, int M, int V, int K,
                       const int* row_draft, float* zd_row, float* part, float* logits, bool force_wide) {
  if (M <= 0) return hipSuccess;
  static const hipError_t attr128 = [] {
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(vocab_kernel<false>),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, CfgVocab::kSmemBytes);
    if (e == hipSuccess)
      e = hipFuncSetAttribute(reinterpret_cast<const void*>(vocab_kernel<true>),
                              hipFuncAttributeMaxDynamicSharedMemorySize, CfgVocab::kSmemBytes);
    return e;
  }();
  if (attr128 != hipSuccess) return attr128;
  const bool stats = row_draft || logits;
  const int MT = (M + 127) / 128, NT = (V + 127) / 128;
  // 256 x 256 tiles once they give every CU two or more (the batched passes); their product is formed with
  // the operand roles swapped, and the draft logits follow suit
  const int MT256 = (M + 255) / 256, NT256 = (V + 255) / 256;
  const bool big = force_wide || (long)MT256 * NT256 >= 512;
  // without row_draft no row scores a draft (drafter pass): every count is taken against -inf, unused
  if (row_draft) {
    if (big) hipLaunchKernelGGL(draft_logit_kernel<true>, dim3((M + 31) / 32), dim3(64), 0, st, A, E, M, V, K, row_draft, zd_row);
    else hipLaunchKernelGGL(draft_logit_kernel<false>, dim3((M + 31) / 32), dim3(64), 0, st, A, E, M, V, K, row_draft, zd_row);
  }
  if (big) {
    constexpr int kSmem256 = CfgVocab256::kSmemBytes;
    static const hipError_t attr256 = [] {
      hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(vocab256_kernel<false>),
                                         hipFuncAttributeMaxDynamicSharedMemorySize, kSmem256);
      if (e == hipSuccess)
        e = hipFuncSetAttribute(reinterpret_cast<const void*>(vocab256_kernel<true>),
                                hipFuncAttributeMaxDynamicSharedMemorySize, kSmem256);
      return e;
    }();
    if (attr256 != hipSuccess) return attr256;
    if (stats)
      SD_LAUNCH_TIMED(vocab256_kernel<false>, dim3(xcd_grid(MT256, NT256)), dim3(CfgVocab256::kThreads), kSmem256, st, A, E, M, V, K, MT256, NT256, NT, row_draft ? zd_row : nullptr, part, logits);
    else
      SD_LAUNCH_TIMED(vocab256_kernel<true>, dim3(xcd_grid(MT256, NT256)), dim3(CfgVocab256::kThreads), kSmem256, st, A, E, M, V, K, MT256, NT256, NT, nullptr, part, logits);
    return hipGetLastError();
  }
  if (stats)
    SD_LAUNCH_TIMED(vocab_kernel<false>, dim3(xcd_grid(MT, NT)), dim3(CfgVocab::kThreads), CfgVocab::kSmemBytes, st,
                       A, E, M, V, K, MT, NT, row_draft ? zd_row : nullptr, part, logits);
  else
    SD_LAUNCH_TIMED(vocab_kernel<true>, dim3(xcd_grid(MT, NT)), dim3(CfgVocab::kThreads), CfgVocab::kSmemBytes, st,
                       A, E, M, V, K, MT, NT, nullptr, part, logits);
  return hipGetLastError();
}

}  // namespace sd
