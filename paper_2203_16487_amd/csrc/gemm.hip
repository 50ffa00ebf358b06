// MFMA GEMM kernels of the decoder / encoder blocks and the fused vocabulary kernel.
#include "gemm_core.h"
#include "kernels.h"

namespace sd {

// ----------------------------------------------------------------------------- epilogues
struct EpiF32 {
  const bf16* bias;
  const float* resid;
  float* out;
  int ldo;
  __device__ __forceinline__ void operator()(int m, int n, float v) const {
    if (bias) v += (float)bias[n];
    size_t o = (size_t)m * ldo + n;
    if (resid) v += resid[o];
    out[o] = v;
  }
};

struct EpiBf16 {
  const bf16* bias;
  bf16* out;
  int ldo;
  int relu;
  __device__ __forceinline__ void operator()(int m, int n, float v) const {
    if (bias) v += (float)bias[n];
    if (relu) v = fmaxf(v, 0.f);
    out[(size_t)m * ldo + n] = (bf16)v;
  }
};

// Decoder self-attention projection: columns [0,d) are queries, [d,2d) keys, [2d,3d) values.
// Keys/values go straight into the cache row of the token they belong to: this is the
// "append" of the KV cache, fused into the projection.
struct EpiQkvAppend {
  const bf16* bias;
  bf16* q;
  bf16* kc;
  bf16* vc;
  const int* row_b;
  const int* row_pos;
  int d, H, Lcap;
  __device__ __forceinline__ void operator()(int m, int n, float v) const {
    v += (float)bias[n];
    int part = n / d, c = n - part * d;
    if (part == 0) {
      q[(size_t)m * d + c] = (bf16)v;
      return;
    }
    int b = row_b[m];
    if (b < 0) return;
    int h = c >> 6, e = c & 63;
    size_t o = (((size_t)b * H + h) * Lcap + row_pos[m]) * kHeadDim + e;
    (part == 1 ? kc : vc)[o] = (bf16)v;
  }
};

struct EpiCrossKv {
  const bf16* bias;
  bf16* xk;
  bf16* xv;
  int d, H, S, Scap;
  __device__ __forceinline__ void operator()(int m, int n, float v) const {
    v += (float)bias[n];
    int part = n / d, c = n - part * d;
    int b = m / S, s = m - b * S;
    int h = c >> 6, e = c & 63;
    size_t o = (((size_t)b * H + h) * Scap + s) * kHeadDim + e;
    (part == 0 ? xk : xv)[o] = (bf16)v;
  }
};

template <class Epi>
__global__ __launch_bounds__(kGemmThreads) void gemm_kernel(const bf16* __restrict__ A, int lda,
                                                            const bf16* __restrict__ W, int ldw,
                                                            int M, int N, int K, Epi epi) {
  __shared__ __attribute__((aligned(16))) bf16 smem[kGemmSmemBytes / 2];
  const int m0 = blockIdx.y * GM, n0 = blockIdx.x * GN;
  GemmAcc acc;
  gemm_mainloop(A, lda, W, ldw, M, N, K, m0, n0, smem, acc);
  gemm_foreach(acc, m0, n0, [&](int m, int n, float v) {
    if (m < M && n < N) epi(m, n, v);
  });
}

template <class Epi>
static hipError_t launch(hipStream_t st, const bf16* A, int lda, const bf16* W, int M, int N, int K,
                         const Epi& epi) {
  if (M <= 0 || N <= 0) return hipSuccess;
  dim3 grid((N + GN - 1) / GN, (M + GM - 1) / GM);
  hipLaunchKernelGGL(gemm_kernel<Epi>, grid, dim3(kGemmThreads), 0, st, A, lda, W, K, M, N, K, epi);
  return hipGetLastError();
}

hipError_t gemm_f32(hipStream_t st, const bf16* A, int lda, const bf16* W, int M, int N, int K,
                    const bf16* bias, const float* resid, float* out, int ldo) {
  return launch(st, A, lda, W, M, N, K, EpiF32{bias, resid, out, ldo});
}
hipError_t gemm_bf16(hipStream_t st, const bf16* A, int lda, const bf16* W, int M, int N, int K,
                     const bf16* bias, bf16* out, int ldo, bool relu) {
  return launch(st, A, lda, W, M, N, K, EpiBf16{bias, out, ldo, relu ? 1 : 0});
}
hipError_t gemm_qkv_append(hipStream_t st, const bf16* A, const bf16* W, int M, int d, int K,
                           const bf16* bias, bf16* q_out, bf16* kc, bf16* vc, const int* row_b,
                           const int* row_pos, int H, int Lcap) {
  return launch(st, A, K, W, M, 3 * d, K, EpiQkvAppend{bias, q_out, kc, vc, row_b, row_pos, d, H, Lcap});
}
hipError_t gemm_cross_kv(hipStream_t st, const bf16* A, const bf16* W, int M, int d, int K,
                         const bf16* bias, bf16* xk, bf16* xv, int S, int H, int Scap) {
  return launch(st, A, K, W, M, 2 * d, K, EpiCrossKv{bias, xk, xv, d, H, S, Scap});
}

// ----------------------------------------------------------------------------- vocabulary
// One block = 128 rows x 128 vocabulary columns.  After the K loop the fp32 tile goes through
// LDS so that two threads own one row (64 columns each); each scans its columns once for
// max / arg-max / top list / draft logit and once for the sum of exponentials, the two halves
// are merged with lane shuffles, and one partial record per (row, tile) is written.  Logits
// never reach memory unless the caller asks for them.
__device__ __forceinline__ int cs_off(int row, int col) {
  // rows r and r+4 are written by the two lane halves of one MFMA register: flip bank half
  return row * GN + (col ^ (((row >> 2) & 1) << 5));
}

__global__ __launch_bounds__(kGemmThreads) void vocab_kernel(const bf16* __restrict__ A,
                                                             const bf16* __restrict__ E, int M,
                                                             int V, int K,
                                                             const int* __restrict__ row_draft,
                                                             float* __restrict__ part,
                                                             float* __restrict__ logits) {
  __shared__ __attribute__((aligned(16))) bf16 smem[kGemmSmemBytes / 2];
  const int m0 = blockIdx.y * GM, n0 = blockIdx.x * GN;
  const int n_tiles = gridDim.x;
  GemmAcc acc;
  gemm_mainloop(A, K, E, K, M, V, K, m0, n0, smem, acc);
  // the main loop ends with a barrier: the staging buffers are free
  float* cs = reinterpret_cast<float*>(smem);  // [128][128] fp32 = 64 KB
  gemm_foreach(acc, 0, 0, [&](int r, int c, float v) { cs[cs_off(r, c)] = v; });
  __syncthreads();

  const int tid = threadIdx.x;
  const int row = tid >> 1, half = tid & 1;
  const int m = m0 + row;
  const int tdraft = (m < M) ? row_draft[m] : -1;
  float best = kNegInf, zd = kNegInf;
  int besti = 0x7fffffff;
  float top[kTopN];
#pragma unroll
  for (int i = 0; i < kTopN; ++i) top[i] = kNegInf;
  // lane (row, half) visits column half*64 + (j + row + 32*half) % 64 at step j: the 64 lanes
  // of a wave hit 64 different banks
  const int rot = row + 32 * half;
  for (int j = 0; j < 64; ++j) {
    int c = half * 64 + ((j + rot) & 63);
    int n = n0 + c;
    float v = cs[cs_off(row, c)];
    if (n < V) {
      if (v > best || (v == best && n < besti)) { best = v; besti = n; }
      top_insert<kTopN>(top, v);
      if (n == tdraft) zd = v;
    }
  }
  float se = 0.f;
  for (int j = 0; j < 64; ++j) {
    int c = half * 64 + ((j + rot) & 63);
    if (n0 + c < V) se += __expf(cs[cs_off(row, c)] - best);
  }
  // merge the two halves of the row (lanes tid and tid^1)
  float obest = __shfl_xor(best, 1, 64);
  int obesti = __shfl_xor(besti, 1, 64);
  float ose = __shfl_xor(se, 1, 64);
  float ozd = __shfl_xor(zd, 1, 64);
  float otop[kTopN];
#pragma unroll
  for (int i = 0; i < kTopN; ++i) otop[i] = __shfl_xor(top[i], 1, 64);
  float nb = fmaxf(best, obest);
  float tot = 0.f;
  if (best > kNegInf) tot += se * __expf(best - nb);
  if (obest > kNegInf) tot += ose * __expf(obest - nb);
  int nbi = (obest > best || (obest == best && obesti < besti)) ? obesti : besti;
#pragma unroll
  for (int i = 0; i < kTopN; ++i) top_insert<kTopN>(top, otop[i]);
  if (half == 0 && m < M) {
    float* p = part + ((size_t)m * n_tiles + blockIdx.x) * kPartF;
    p[0] = nb;
    p[1] = __int_as_float(nbi);
    p[2] = tot;
    p[3] = fmaxf(zd, ozd);
#pragma unroll
    for (int i = 0; i < kTopN; ++i) p[4 + i] = top[i];
  }
  if (logits) {
    for (int idx = tid; idx < GM * GN; idx += kGemmThreads) {
      int r = idx >> 7, c = idx & 127;
      if (m0 + r < M && n0 + c < V) logits[(size_t)(m0 + r) * V + n0 + c] = cs[cs_off(r, c)];
    }
  }
}

hipError_t vocab_stats(hipStream_t st, const bf16* A, const bf16* E, int M, int V, int K,
                       const int* row_draft, float* part, float* logits) {
  if (M <= 0) return hipSuccess;
  dim3 grid((V + GN - 1) / GN, (M + GM - 1) / GM);
  hipLaunchKernelGGL(vocab_kernel, grid, dim3(kGemmThreads), 0, st, A, E, M, V, K, row_draft, part,
                     logits);
  return hipGetLastError();
}

}  // namespace sd
