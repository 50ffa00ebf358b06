// 128x128x64 bf16 "NT" GEMM main loop on MFMA 32x32x16 (gfx950), fp32 accumulation.
//   C[m][n] = sum_k A[m][k] * W[n][k]      A [M,K] row-major (lda), W [N,K] row-major (ldw)
// Both operands are K-contiguous, which is how activations and nn-style weights lie in
// memory, so every global load is a 16-byte row segment and every MFMA operand is one
// 16-byte LDS read.  256 threads = 4 waves in a 2x2 arrangement, 64x64 outputs per wave.
#pragma once
#include "common.h"

namespace sd {

constexpr int GM = 128, GN = 128, GK = 64;
constexpr int kGemmThreads = 256;
constexpr int kTileElems = 128 * GK;                 // bf16 elements of one operand tile
constexpr int kGemmSmemBytes = 2 * 2 * kTileElems * 2;  // double-buffered A and W tiles (64 KB)

// LDS tile: 128 rows of 64 bf16 (8 chunks of 16 B).  Chunk c of row r lives at chunk
// c ^ ((r >> 1) & 7): 16 consecutive rows reading the same logical chunk then touch all
// 64 banks exactly once, and so does a 16-lane group writing two full rows.
__device__ __forceinline__ int lds_off(int row, int chunk) {
  return row * GK + ((chunk ^ ((row >> 1) & 7)) << 3);
}

struct GemmAcc {
  f32x16 c[2][2];  // [m-tile][n-tile] of the wave's 64x64 block
};

// Runs the whole K loop for the block tile at (m0, n0).  Rows >= M / >= N read as zero.
// K must be a multiple of 64; lda, ldw multiples of 8; A, W 16-byte aligned.
__device__ __forceinline__ void gemm_mainloop(const bf16* __restrict__ A, int lda,
                                              const bf16* __restrict__ W, int ldw, int M, int N,
                                              int K, int m0, int n0, bf16* smem, GemmAcc& acc) {
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wm = (wave >> 1) * 64, wn = (wave & 1) * 64;
#pragma unroll
  for (int i = 0; i < 2; ++i)
#pragma unroll
    for (int j = 0; j < 2; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc.c[i][j][r] = 0.f;

  // this thread's four 16-byte segments of each operand tile
  const uint4* ga[4];
  const uint4* gw[4];
  int so[4];
  bool oka[4], okw[4];
#pragma unroll
  for (int p = 0; p < 4; ++p) {
    int idx = p * 256 + tid, row = idx >> 3, ch = idx & 7;
    so[p] = lds_off(row, ch);
    oka[p] = (m0 + row) < M;
    okw[p] = (n0 + row) < N;
    ga[p] = reinterpret_cast<const uint4*>(A + (size_t)(oka[p] ? m0 + row : 0) * lda + ch * 8);
    gw[p] = reinterpret_cast<const uint4*>(W + (size_t)(okw[p] ? n0 + row : 0) * ldw + ch * 8);
  }
  const uint4 zero4 = make_uint4(0, 0, 0, 0);
  uint4 ra[4], rw[4];
#pragma unroll
  for (int p = 0; p < 4; ++p) {
    ra[p] = oka[p] ? ga[p][0] : zero4;
    rw[p] = okw[p] ? gw[p][0] : zero4;
  }
  bf16* sA = smem;                    // [2][kTileElems]
  bf16* sW = smem + 2 * kTileElems;   // [2][kTileElems]
#pragma unroll
  for (int p = 0; p < 4; ++p) {
    *reinterpret_cast<uint4*>(sA + so[p]) = ra[p];
    *reinterpret_cast<uint4*>(sW + so[p]) = rw[p];
  }
  __syncthreads();

  const int KT = K / GK;
  const int lrow = lane & 31, lhalf = lane >> 5;
  for (int kt = 0; kt < KT; ++kt) {
    const int cur = kt & 1;
    if (kt + 1 < KT) {
#pragma unroll
      for (int p = 0; p < 4; ++p) {   // 8 bf16 per uint4 -> advance by 8 uint4 per 64-k step
        ra[p] = oka[p] ? ga[p][(kt + 1) * 8] : zero4;
        rw[p] = okw[p] ? gw[p][(kt + 1) * 8] : zero4;
      }
    }
    const bf16* cA = sA + cur * kTileElems;
    const bf16* cW = sW + cur * kTileElems;
#pragma unroll
    for (int kk = 0; kk < 4; ++kk) {
      bf16x8 a[2], b[2];
#pragma unroll
      for (int i = 0; i < 2; ++i)
        a[i] = *reinterpret_cast<const bf16x8*>(cA + lds_off(wm + i * 32 + lrow, kk * 2 + lhalf));
#pragma unroll
      for (int j = 0; j < 2; ++j)
        b[j] = *reinterpret_cast<const bf16x8*>(cW + lds_off(wn + j * 32 + lrow, kk * 2 + lhalf));
#pragma unroll
      for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j)
          acc.c[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[i], b[j], acc.c[i][j], 0, 0, 0);
    }
    if (kt + 1 < KT) {
      bf16* nA = sA + (cur ^ 1) * kTileElems;
      bf16* nW = sW + (cur ^ 1) * kTileElems;
#pragma unroll
      for (int p = 0; p < 4; ++p) {
        *reinterpret_cast<uint4*>(nA + so[p]) = ra[p];
        *reinterpret_cast<uint4*>(nW + so[p]) = rw[p];
      }
    }
    __syncthreads();
  }
}

// Visits every output element the calling lane holds: f(m, n, value).
// MFMA 32x32 result layout: register r of lane l is row 8*(r/4) + 4*(l/32) + r%4, col l%32.
template <class F>
__device__ __forceinline__ void gemm_foreach(const GemmAcc& acc, int m0, int n0, F&& f) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int wm = (wave >> 1) * 64, wn = (wave & 1) * 64;
#pragma unroll
  for (int i = 0; i < 2; ++i)
#pragma unroll
    for (int j = 0; j < 2; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        int m = m0 + wm + i * 32 + 8 * (r >> 2) + 4 * (lane >> 5) + (r & 3);
        int n = n0 + wn + j * 32 + (lane & 31);
        f(m, n, acc.c[i][j][r]);
      }
}

}  // namespace sd
