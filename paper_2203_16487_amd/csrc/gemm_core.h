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
#include <stdint.h>

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

// Global -> LDS request of 64 lanes x 16 bytes, landing at lds_dst + lane * 16 (lds_dst is the same
// for the whole wave).  An asm statement, so that the compiler does not order it against the LDS
// reads in flight (it would wait for all of them before every request); the ring protocol of the
// main loop guarantees that the slot being filled is not read between the two barriers around the
// request.  The compiler's own vmcnt bookkeeping stays safe: loads complete in order, and a count it
// computes without these requests can only make it wait longer.
__device__ __forceinline__ void dma16(const bf16* g, bf16* lds_dst) {
  const unsigned l = __builtin_amdgcn_readfirstlane((unsigned)(uintptr_t)SD_LDS_PTR(lds_dst));
  asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, off" ::"s"(l), "v"(g));
}

// wait until at most allow * IPW of this wave's requests are outstanding (allow in [0, MAXA])
template <int IPW, int MAXA>
__device__ __forceinline__ void wait_vm_stages(int allow) {
  if constexpr (MAXA <= 0) {
    wait_vmcnt<0>();
  } else {
    if (allow >= MAXA) wait_vmcnt<IPW * MAXA>();
    else wait_vm_stages<IPW, MAXA - 1>(allow);
  }
}

// Whole K range [k_begin, k_begin + GK*KT) of the block tile at (m0, n0).  Rows beyond M / N
// are clamped to the last valid row (their products land in outputs that are never stored).
// Requirements: K % GK == 0, lda/ldw % 8 == 0, A and W 16-byte aligned, smem 1024-aligned.
//
// Stage j (GK columns of k) lives in ring slot j % S and is multiplied in GK/16 sub-steps of one
// MFMA per 32x32 tile each.  What keeps the matrix pipe busy:
//  * the fragments of sub-step s+1 are read from LDS into a second register set while the MFMAs
//    of sub-step s issue, in a fixed order written out in the source (MFMA, LDS read, MFMA, ...);
//  * the block's one barrier per stage sits before the LAST sub-step of stage kt and certifies
//    that stage kt+1 has landed for every wave, so the fragments of (kt+1, 0) are read while the
//    last MFMAs of stage kt run: no wave ever waits for LDS latency right after a barrier;
//  * with S >= 3 the requests of stage kt+S-1 (slot of stage kt-1, free since the barrier inside
//    stage kt-1) go out a few per sub-step during stage kt instead of in one burst; with S = 2
//    the requests of stage kt+2 follow the barrier inside stage kt (the slot just vacated).
// SWAP: W rows take the MFMA's row operand and A rows its column operand: register r of lane l of
// tile (i, j) then holds row m = 32 i + l%32, column n = 32 j + 8*(r/4) + 4*(l/32) + r%4 (relative to
// the wave tile), i.e. a lane owns 16 columns of ONE row per tile instead of 16 rows of one column.
template <class Cfg, bool SWAP = false>
__device__ __forceinline__ void gemm_mainloop(const bf16* __restrict__ A, int lda,
                                              const bf16* __restrict__ W, int ldw, int M, int N,
                                              int k_begin, int KT, int m0, int n0, bf16* smem,
                                              GemmAcc<Cfg>& acc) {
  constexpr int IPW = Cfg::kIPW, S = Cfg::kStages, GK = Cfg::GK, RPL = Cfg::kRowsPerLoad, CPR = GK / 8;
  constexpr int TM = Cfg::kTM, TN = Cfg::kTN, NS = GK / 16, TMIN = TM < TN ? TM : TN;
  static_assert(S >= 2 && NS % 2 == 0, "ring depth / fragment buffer parity");
  constexpr bool SPREAD = S >= 3;
  constexpr int PRO = SPREAD ? S - 1 : S;      // stages requested before the loop
  constexpr int AHEAD = PRO;                   // during stage kt the requests of stage kt + AHEAD go out
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wm = (wave / Cfg::kWavesN) * Cfg::kWM, wn = (wave % Cfg::kWavesN) * Cfg::kWN;
#pragma unroll
  for (int i = 0; i < TM; ++i)
#pragma unroll
    for (int j = 0; j < TN; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc.c[i][j][r] = 0.f;

  // One request moves 64 lanes x 16 B = RPL tile rows; lane l lands at row l/CPR, physical chunk
  // l%CPR, so it fetches the logical chunk that the swizzle maps there.
  const bf16* gptr[IPW];
#pragma unroll
  for (int i = 0; i < IPW; ++i) {
    const int row = (wave * IPW + i) * RPL + lane / CPR;
    const int chunk = GK == 64 ? ((lane & 7) ^ ((row >> 1) & 7)) : ((lane & 3) ^ ((row >> 2) & 3));
    if (row < Cfg::kBM) gptr[i] = A + (size_t)min(m0 + row, M - 1) * lda + k_begin + chunk * 8;
    else gptr[i] = W + (size_t)min(n0 + row - Cfg::kBM, N - 1) * ldw + k_begin + chunk * 8;
  }
  bf16* const wslot = smem + wave * IPW * 512;   // this wave's part of slot 0
#pragma unroll
  for (int s = 0; s < PRO; ++s)
    if (s < KT) {
#pragma unroll
      for (int i = 0; i < IPW; ++i) dma16(gptr[i] + s * GK, wslot + s * Cfg::kStageElems + i * 512);
    }
  const int lrow = lane & 31, lhalf = lane >> 5;
  int offA[TM][NS], offB[TN][NS];   // fragment offsets inside a stage
#pragma unroll
  for (int ss = 0; ss < NS; ++ss) {
#pragma unroll
    for (int i = 0; i < TM; ++i) offA[i][ss] = lds_off<GK>(wm + i * 32 + lrow, ss * 2 + lhalf);
#pragma unroll
    for (int j = 0; j < TN; ++j) offB[j][ss] = Cfg::kBM * GK + lds_off<GK>(wn + j * 32 + lrow, ss * 2 + lhalf);
  }
  bf16x8 fa[2][TM], fb[2][TN];
  // fragment q of a sub-step in read order a0 b0 a1 b1 ..: the first product of the next sub-step
  // gets its operands first
  auto read_frag = [&](int buf, const bf16* st, int ss, int q) {
    const bool isA = q < 2 * TMIN ? (q & 1) == 0 : TM > TN;
    const int idx = q < 2 * TMIN ? q >> 1 : q - TMIN;
    if (isA) fa[buf][idx] = *reinterpret_cast<const bf16x8*>(st + offA[idx][ss]);
    else fb[buf][idx] = *reinterpret_cast<const bf16x8*>(st + offB[idx][ss]);
  };
  // One sub-step in issue order.  cur: fragment set multiplied now; READ: the fragments of
  // (nst, nss) go to the other set; requests [d0, d1) of stage dkt go to slot dslot.
  auto substep = [&](int cur, bool READ, const bf16* nst, int nss, int dkt, int dslot, int d0, int d1) {
    int nread = 0, nd = d0;
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
      for (int j = 0; j < TN; ++j) {
        acc.c[i][j] = SWAP ? __builtin_amdgcn_mfma_f32_32x32x16_bf16(fb[cur][j], fa[cur][i], acc.c[i][j], 0, 0, 0)
                           : __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[cur][i], fb[cur][j], acc.c[i][j], 0, 0, 0);
        if (READ && nread < TM + TN) read_frag(cur ^ 1, nst, nss, nread++);
        if (((i * TN + j) & 1) && nd < d1) {
          dma16(gptr[nd] + dkt * GK, wslot + dslot * Cfg::kStageElems + nd * 512);
          ++nd;
        }
        __builtin_amdgcn_sched_barrier(0);
      }
    if (READ) {   // fewer products than fragments
#pragma unroll
      for (; nread < TM + TN; ++nread) read_frag(cur ^ 1, nst, nss, nread);
    }
#pragma unroll
    for (; nd < d1; ++nd) dma16(gptr[nd] + dkt * GK, wslot + dslot * Cfg::kStageElems + nd * 512);
  };
  // stage 0 has landed for everyone
  wait_vm_stages<IPW, PRO - 1>(min(PRO, KT) - 1);
  block_barrier();
#pragma unroll
  for (int q = 0; q < TM + TN; ++q) read_frag(0, smem, 0, q);
  constexpr int LASTBUF = (NS - 1) & 1;
  int kt = 0;
  // stages during which another stage is still to be requested
  for (; kt + AHEAD < KT; ++kt) {
    const bf16* st = smem + (kt % S) * Cfg::kStageElems;
    const int nslot = (kt + AHEAD) % S;
#pragma unroll
    for (int ss = 0; ss + 1 < NS; ++ss)
      substep(ss & 1, true, st, ss + 1, kt + AHEAD, nslot, SPREAD ? ss * IPW / NS : 0, SPREAD ? (ss + 1) * IPW / NS : 0);
    // my reads of this stage are done (its slot may be refilled after the barrier), my part of
    // stage kt+1 has landed (younger requests may still be in flight)
    asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
    wait_vmcnt<SPREAD ? IPW * (S - 3) + (NS - 1) * IPW / NS : IPW * (S - 2)>();
    block_barrier();
    __builtin_amdgcn_sched_barrier(0);
    substep(LASTBUF, true, smem + ((kt + 1) % S) * Cfg::kStageElems, 0, kt + AHEAD, nslot,
            SPREAD ? (NS - 1) * IPW / NS : 0, IPW);
  }
  // the last stages: nothing left to request
  for (; kt + 1 < KT; ++kt) {
    const bf16* st = smem + (kt % S) * Cfg::kStageElems;
#pragma unroll
    for (int ss = 0; ss + 1 < NS; ++ss) substep(ss & 1, true, st, ss + 1, 0, 0, 0, 0);
    asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
    wait_vm_stages<IPW, AHEAD - 2>(KT - kt - 2);
    block_barrier();
    __builtin_amdgcn_sched_barrier(0);
    substep(LASTBUF, true, smem + ((kt + 1) % S) * Cfg::kStageElems, 0, 0, 0, 0, 0);
  }
  {
    const bf16* st = smem + (kt % S) * Cfg::kStageElems;
#pragma unroll
    for (int ss = 0; ss + 1 < NS; ++ss) substep(ss & 1, true, st, ss + 1, 0, 0, 0, 0);
    substep(LASTBUF, false, st, 0, 0, 0, 0, 0);
  }
#pragma unroll
  for (int i = 0; i < TM; ++i)
#pragma unroll
    for (int j = 0; j < TN; ++j) mfma_settle(acc.c[i][j]);
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
