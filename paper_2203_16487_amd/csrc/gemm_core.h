// bf16 "NT" GEMM main loop on MFMA 32x32x16 (gfx950), fp32 accumulation.
//   C[m][n] = sum_k A[m][k] * W[n][k]      A [M,K] row-major (lda), W [N,K] row-major (ldw)
// Both operands are K-contiguous (activations and nn-style weights), so every global access
// is a 16-byte row segment and every MFMA operand is one 16-byte LDS read.
//
// Tiles of BM x BN x 64 move from global memory straight into LDS (global_load_lds, 16 bytes
// per lane, no register staging) through a ring of STAGES buffers, so that STAGES-1 tiles of
// loads are in flight while one is being multiplied: HBM/L2 latency (~1-2 us) is covered by
// depth, not by occupancy.  Waves form a WAVES_M x WAVES_N arrangement (4 or 8 waves).
#pragma once
#include "common.h"

namespace sd {

constexpr int kGemmThreads = 256;


template <int N>
__device__ __forceinline__ void wait_vmcnt() {
  asm volatile("s_waitcnt vmcnt(%0)" ::"n"(N) : "memory");
}
// Workgroup barrier without the release/acquire fences of __syncthreads(): those would wait
// for every outstanding global_load_lds (vmcnt(0)) and flatten the pipeline.  The memory
// clobber keeps the compiler from moving LDS accesses across it.
__device__ __forceinline__ void block_barrier() { asm volatile("s_barrier" ::: "memory"); }

// LDS tile rows hold GK bf16 (the k extent of one pipeline stage) = GK/8 chunks of 16 B.
// GK = 64: chunk c of row r lives at chunk c ^ ((r >> 1) & 7); GK = 32: at c ^ ((r >> 2) & 3).
// Either way 16 consecutive rows reading the same logical chunk touch all 64 banks once.
template <int GK>
__device__ __forceinline__ int lds_off(int row, int chunk) {
  static_assert(GK == 64 || GK == 32, "stage depth");
  return GK == 64 ? row * 64 + ((chunk ^ ((row >> 1) & 7)) << 3) : row * 32 + ((chunk ^ ((row >> 2) & 3)) << 3);
}

template <int BM, int BN, int STAGES, int WAVES_M = 2, int WAVES_N = 2, int GK_ = 64>
struct GemmCfg {
  static constexpr int GK = GK_;
  static constexpr int kRowsPerLoad = 512 / GK;        // tile rows moved by one global_load_lds
  static constexpr int kBM = BM, kBN = BN, kStages = STAGES;
  static constexpr int kWavesM = WAVES_M, kWavesN = WAVES_N, kWaves = WAVES_M * WAVES_N;
  static constexpr int kThreads = 64 * kWaves;
  static constexpr int kRows = BM + BN;                 // LDS rows per stage (A rows then W rows)
  static constexpr int kIPW = kRows / kRowsPerLoad / kWaves;   // global_load_lds per wave per stage
  static constexpr int kStageElems = kRows * GK;
  static constexpr int kSmemBytes = STAGES * kStageElems * 2;
  static constexpr int kWM = BM / WAVES_M, kWN = BN / WAVES_N;   // wave tile
  static constexpr int kTM = kWM / 32, kTN = kWN / 32;           // MFMA tiles per wave
  static_assert(kRows % (kRowsPerLoad * kWaves) == 0 && BM % kRowsPerLoad == 0 && kWM % 32 == 0 && kWN % 32 == 0,
                "tile shape");
};

template <class Cfg>
struct GemmAcc {
  f32x16 c[Cfg::kTM][Cfg::kTN];
};

template <class Cfg>
struct GemmFrag {
  bf16x8 a[Cfg::kTM], b[Cfg::kTN];
};

template <class Cfg>
__device__ __forceinline__ void load_frags(GemmFrag<Cfg>& f, const bf16* sA, const bf16* sW, int wm,
                                           int wn, int lrow, int lhalf, int kk) {
#pragma unroll
  for (int i = 0; i < Cfg::kTM; ++i)
    f.a[i] = *reinterpret_cast<const bf16x8*>(sA + lds_off<Cfg::GK>(wm + i * 32 + lrow, kk * 2 + lhalf));
#pragma unroll
  for (int j = 0; j < Cfg::kTN; ++j)
    f.b[j] = *reinterpret_cast<const bf16x8*>(sW + lds_off<Cfg::GK>(wn + j * 32 + lrow, kk * 2 + lhalf));
}

template <class Cfg>
__device__ __forceinline__ void mma_frags(GemmAcc<Cfg>& acc, const GemmFrag<Cfg>& f) {
#pragma unroll
  for (int i = 0; i < Cfg::kTM; ++i)
#pragma unroll
    for (int j = 0; j < Cfg::kTN; ++j)
      acc.c[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(f.a[i], f.b[j], acc.c[i][j], 0, 0, 0);
}

// Whole K range [k_begin, k_begin + GK*KT) of the block tile at (m0, n0).  Rows beyond M / N
// are clamped to the last valid row (their products land in outputs that are never stored).
// Requirements: K % GK == 0, lda/ldw % 8 == 0, A and W 16-byte aligned, smem 1024-aligned.
template <class Cfg>
__device__ __forceinline__ void gemm_mainloop(const bf16* __restrict__ A, int lda,
                                              const bf16* __restrict__ W, int ldw, int M, int N,
                                              int k_begin, int KT, int m0, int n0, bf16* smem,
                                              GemmAcc<Cfg>& acc) {
  constexpr int IPW = Cfg::kIPW, STAGES = Cfg::kStages, GK = Cfg::GK, RPL = Cfg::kRowsPerLoad, CPR = GK / 8;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wm = (wave / Cfg::kWavesN) * Cfg::kWM, wn = (wave % Cfg::kWavesN) * Cfg::kWN;
#pragma unroll
  for (int i = 0; i < Cfg::kTM; ++i)
#pragma unroll
    for (int j = 0; j < Cfg::kTN; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc.c[i][j][r] = 0.f;

  // One global_load_lds moves 64 lanes x 16 B = RPL tile rows; lane l lands at row l/CPR,
  // physical chunk l%CPR, so it fetches the logical chunk that the swizzle maps there.
  const bf16* gptr[IPW];
#pragma unroll
  for (int i = 0; i < IPW; ++i) {
    const int row = (wave * IPW + i) * RPL + lane / CPR;
    const int chunk = GK == 64 ? ((lane & 7) ^ ((row >> 1) & 7)) : ((lane & 3) ^ ((row >> 2) & 3));
    if (row < Cfg::kBM) {
      gptr[i] = A + (size_t)min(m0 + row, M - 1) * lda + k_begin + chunk * 8;
    } else {
      gptr[i] = W + (size_t)min(n0 + row - Cfg::kBM, N - 1) * ldw + k_begin + chunk * 8;
    }
  }
  auto issue = [&](int kt, int slot) {
#pragma unroll
    for (int i = 0; i < IPW; ++i) {
      bf16* dst = smem + slot * Cfg::kStageElems + (wave * IPW + i) * 512;
      __builtin_amdgcn_global_load_lds(SD_GLB_PTR(gptr[i] + kt * GK), SD_LDS_PTR(dst), 16, 0, 0);
    }
  };
#pragma unroll
  for (int s = 0; s < STAGES - 1; ++s)
    if (s < KT) issue(s, s);

  const int lrow = lane & 31, lhalf = lane >> 5;
  for (int kt = 0; kt < KT; ++kt) {
    // tile kt has landed once at most STAGES-2 younger tiles are still in flight
    if (kt + STAGES - 2 < KT) wait_vmcnt<IPW * (STAGES - 2)>(); else wait_vmcnt<0>();
    block_barrier();   // everyone's part of tile kt is in LDS; everyone is done with tile kt-1
    if (kt + STAGES - 1 < KT) issue(kt + STAGES - 1, (kt + STAGES - 1) % STAGES);
    const bf16* sA = smem + (kt % STAGES) * Cfg::kStageElems;
    const bf16* sW = sA + Cfg::kBM * GK;
    // fragments of step kk+1 are fetched from LDS while the MFMAs of step kk run
    GemmFrag<Cfg> f0, f1;
    load_frags<Cfg>(f0, sA, sW, wm, wn, lrow, lhalf, 0);
    load_frags<Cfg>(f1, sA, sW, wm, wn, lrow, lhalf, 1);
    mma_frags<Cfg>(acc, f0);
    if (GK == 64) {
      load_frags<Cfg>(f0, sA, sW, wm, wn, lrow, lhalf, 2);
      mma_frags<Cfg>(acc, f1);
      load_frags<Cfg>(f1, sA, sW, wm, wn, lrow, lhalf, 3);
      mma_frags<Cfg>(acc, f0);
    }
    mma_frags<Cfg>(acc, f1);
  }
#pragma unroll
  for (int i = 0; i < Cfg::kTM; ++i)
#pragma unroll
    for (int j = 0; j < Cfg::kTN; ++j) mfma_settle(acc.c[i][j]);
  block_barrier();   // LDS may be reused by the caller's epilogue
}

// Visits every output element the calling lane holds: f(m, n, value).
// MFMA 32x32 result layout: register r of lane l is row 8*(r/4) + 4*(l/32) + r%4, col l%32.
template <class Cfg, class F>
__device__ __forceinline__ void gemm_foreach(const GemmAcc<Cfg>& acc, int m0, int n0, F&& f) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int wm = (wave / Cfg::kWavesN) * Cfg::kWM, wn = (wave % Cfg::kWavesN) * Cfg::kWN;
#pragma unroll
  for (int i = 0; i < Cfg::kTM; ++i)
#pragma unroll
    for (int j = 0; j < Cfg::kTN; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        int m = m0 + wm + i * 32 + 8 * (r >> 2) + 4 * (lane >> 5) + (r & 3);
        int n = n0 + wn + j * 32 + (lane & 31);
        f(m, n, acc.c[i][j][r]);
      }
}

}  // namespace sd
