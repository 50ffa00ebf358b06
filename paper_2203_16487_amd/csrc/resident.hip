// Verification pass of at most 32 rows as ONE resident kernel (Sec. 2; Sec. 3.2).
//
// With so few rows the pass is a chain of ~6 dependent weight-streaming products per layer and
// its cost is the hand-over between them: as separate kernels each hand-over is a kernel
// boundary (launch + the consumer's first read of data another XCD wrote, ~5 us together).
// Here kRsWorkers workgroups stay resident for the whole pass and hand over through a grid
// barrier (~1.5 us including the consumer's read):
//   * every value one workgroup produces for another (residual sums, Q, appended K/V rows, FFN
//     hidden) is stored and loaded with device-scope relaxed atomics (st_coh / ld_coh), which
//     are coherent across XCDs without writing back or invalidating the L2s;
//   * a workgroup arrives at the barrier after s_waitcnt vmcnt(0) (its stores are acknowledged)
//     with one relaxed device-scope increment; one thread per workgroup polls the counter.
// The wait is bounded: after kRsSpinMax polls a workgroup raises the error flag, every
// workgroup leaves at its next poll, and the kernel returns with the flag set (the host
// reports accept_len = -1).  All kRsWorkers workgroups are co-resident by construction
// (32 workgroups of 256 threads on 256 CUs, launched on an in-order stream).
//
// Phases per layer (a barrier after each): QKV + append | self-attention + O | cross Q |
// cross-attention + O | FFN1 | FFN2; then the vocabulary tiles.  A workgroup owns the 16-column
// output slices vb = w, w + 32, ... of each product, recomputes the LayerNorm prologue once
// per phase, and (attention phases) recomputes the attention of every head redundantly, as the
// per-projection kernels do.
#include <hip/hip_runtime.h>

#include <type_traits>

#include "skinny_core.h"

namespace sd {

constexpr unsigned kRsSpinMax = 1u << 20;
constexpr int kRsHelpers = 224;   // most workgroups that only do vocabulary tiles
constexpr int kRsFlagPitch = 64;  // words between two helpers' wake-up words (256 bytes)


struct RsState {
  unsigned* cnt;      // arrival counter of this launch
  unsigned* err;      // error flag (sticky)
  unsigned target;    // thread 0: arrivals that complete the next barrier
  int* flag;          // LDS: outcome of the latest barrier
};

// The barrier comes in two halves so that work that does not depend on other workgroups (the
// next phase's weight requests) can sit between them: rs_arrive publishes this workgroup's
// stores, rs_wait returns once every workgroup has arrived; false = abandon the pass.
__device__ __forceinline__ void rs_arrive(RsState& b) {
  asm volatile("s_waitcnt vmcnt(0)" ::: "memory");   // this thread's stores are acknowledged
  __syncthreads();
  if (threadIdx.x == 0) {
    b.target += kRsWorkers;
    __hip_atomic_fetch_add(b.cnt, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  }
}
__device__ __forceinline__ bool rs_wait(RsState& b) {
  if (threadIdx.x == 0) {
    unsigned spins = 0;
    int bad = 0;
    while (__hip_atomic_load(b.cnt, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) < b.target) {
      if (++spins > kRsSpinMax || __hip_atomic_load(b.err, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) != 0u) {
        __hip_atomic_store(b.err, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        bad = 1;
        break;
      }
      __builtin_amdgcn_s_sleep(1);
    }
    *b.flag = bad;
  }
  // workgroup barrier that does not wait for the weight requests in flight (__syncthreads would)
  asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");
  return *b.flag == 0;
}

// ---- phases --------------------------------------------------------------------------------
// Weights do not depend on the pass, so a workgroup requests the slices it needs in phase p + 1
// right after the products of phase p and holds them in registers (`pre`, 64 VGPRs) across the
// barrier: the HBM latency of cold weights (~2 us) is off the critical path.
constexpr int kRsPre = 16;

template <int PER, int N>   // projection with K = d and N output columns (N % 16 == 0)
struct RsProj {
  static constexpr int d = 64 * PER, S = d / 128, nvb = N / 16;
  static constexpr int NSL = (nvb + kRsWorkers - 1) / kRsWorkers;          // slices per workgroup
  static constexpr int NPF = (kRsPre / S < NSL) ? kRsPre / S : NSL;        // of which held in `pre`
};

// slices i < NPF of projection W [N][K] for workgroup w: this wave's k range [k0, k0 + 32*S)
template <int S, int NPF>
__device__ __forceinline__ void rs_prefetch(bf16x8 (&pre)[kRsPre], const bf16* __restrict__ W, int ldw, int N,
                                            int nvb, int k0, int w) {
  const int lane = threadIdx.x & 63, lq = lane & 15, g = lane >> 4;
#pragma unroll
  for (int i = 0; i < NPF; ++i) {
    const int vb = w + kRsWorkers * i;
    if (vb < nvb) {
      const bf16* wp = W + (size_t)min(vb * 16 + lq, N - 1) * ldw + k0 + 8 * g;
#pragma unroll
      for (int u = 0; u < S; ++u) pre[i * S + u] = *reinterpret_cast<const bf16x8*>(wp + u * 32);
    }
  }
}
template <int PER, int N>
__device__ __forceinline__ void rs_prefetch_proj(bf16x8 (&pre)[kRsPre], const bf16* __restrict__ W, int w) {
  using P = RsProj<PER, N>;
  rs_prefetch<P::S, P::NPF>(pre, W, P::d, N, P::nvb, (threadIdx.x >> 6) * (P::d / 4), w);
}
template <int PER, int FS>   // FFN2: K = F = 128*FS, N = d; first kSkW steps of the first slice
__device__ __forceinline__ void rs_prefetch_ffn2(bf16x8 (&pre)[kRsPre], const bf16* __restrict__ W, int w) {
  constexpr int d = 64 * PER, F = 128 * FS, S1 = FS < kSkW ? FS : kSkW;
  rs_prefetch<S1, 1>(pre, W, F, d, d / 16, (threadIdx.x >> 6) * (F / 4), w);
}

// slice i of a K = d projection: acc += W-slice . hidden (hb in LDS)
template <int PER, int N, bool TWO, int I, class GetB>
__device__ __forceinline__ void rs_slice_mma(const bf16x8 (&pre)[kRsPre], const bf16* __restrict__ W, int vb, int k0,
                                             GetB&& getB, f32x4 (&acc)[2]) {
  using P = RsProj<PER, N>;
  sk_zero(acc);
  if constexpr (I < P::NPF) {
    const int g = (threadIdx.x & 63) >> 4;
#pragma unroll
    for (int u = 0; u < P::S; ++u) {
      const int k = k0 + u * 32 + 8 * g;
      acc[0] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(pre[I * P::S + u], getB(0, k), acc[0], 0, 0, 0);
      if (TWO) acc[1] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(pre[I * P::S + u], getB(1, k), acc[1], 0, 0, 0);
    }
    mfma_settle(acc[0], acc[1]);
  } else {
    bf16x8 wf[P::S];
    sk_wload<P::S>(W, P::d, vb * 16, N, k0, wf);
    sk_mma<P::S, TWO>(wf, k0, getB, acc);
  }
}

// out columns of  hidden(src) W^T  for the slices of workgroup w; epi(m, n, value)
template <int PER, int N, bool TWO, class Epi>
__device__ __forceinline__ void rs_project(const SkLds<PER>& L, const SkSrc& src, int R, const bf16* __restrict__ W,
                                           int w, const bf16x8 (&pre)[kRsPre], Epi&& epi) {
  using P = RsProj<PER, N>;
  constexpr int pitch = P::d + kSkPad;
  const int wave = threadIdx.x >> 6, lq = threadIdx.x & 15;
  const int k0 = wave * (P::d / 4);
  if (w >= P::nvb) return;
  sk_hidden<PER, true>(src, R, TWO ? 32 : 16, L.hb, L.hown, -64, true);
  __syncthreads();
  const bf16* hb = L.hb;
  auto getB = [&](int t, int k) { return *reinterpret_cast<const bf16x8*>(hb + (t * 16 + lq) * pitch + k); };
  auto slice = [&](auto ic) {
    constexpr int I = decltype(ic)::value;
    const int vb = w + kRsWorkers * I;
    if (vb >= P::nvb) return;
    f32x4 acc[2];
    rs_slice_mma<PER, N, TWO, I>(pre, W, vb, k0, getB, acc);
    const int n0 = vb * 16;
    sk_reduce(acc, L.red, R, [&](int m, int nl, float v) { epi(m, n0 + nl, v); });
    __syncthreads();   // red is reused by the next slice
  };
  static_assert(P::NSL <= 8, "slices per workgroup");
  slice(std::integral_constant<int, 0>{});
  if constexpr (P::NSL > 1) slice(std::integral_constant<int, 1>{});
  if constexpr (P::NSL > 2) slice(std::integral_constant<int, 2>{});
  if constexpr (P::NSL > 3) slice(std::integral_constant<int, 3>{});
  if constexpr (P::NSL > 4) slice(std::integral_constant<int, 4>{});
  if constexpr (P::NSL > 5) slice(std::integral_constant<int, 5>{});
  if constexpr (P::NSL > 6) slice(std::integral_constant<int, 6>{});
  if constexpr (P::NSL > 7) slice(std::integral_constant<int, 7>{});
}

// xs_out = hidden(resid) + attention(all heads) Wo^T + bias
template <int PER, bool VBLK, bool TWO>
__device__ __forceinline__ void rs_attn_o(const SkLds<PER>& L, const SkSrc& resid, int R, const AttnArgs& a,
                                          const bf16* __restrict__ W, const bf16* __restrict__ bias,
                                          float* xs_out, int w, const bf16x8 (&pre)[kRsPre]) {
  constexpr int d = 64 * PER, pitch = d + kSkPad;
  using P = RsProj<PER, d>;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, lq = lane & 15, g = lane >> 4;
  const int k0 = wave * (d / 4);
  if (w >= P::nvb) return;
  const int vb1 = w + kRsWorkers;                     // second slice of this workgroup (d = 1024)
  sk_hidden<PER, true>(resid, R, TWO ? 32 : 16, L.hb, L.hown, w * 16, false, vb1 < P::nvb ? vb1 * 16 : -64);
  for (int idx = threadIdx.x; idx < (TWO ? 32 : 16) * pitch / 8; idx += kSkThreads)
    reinterpret_cast<uint4*>(L.hb)[idx] = make_uint4(0, 0, 0, 0);
  __syncthreads();
  for (int p = wave; p < a.B * a.H; p += 4) {
    const int b = p / a.H, h = p - b * a.H;
    constexpr int NQT = TWO ? 2 : 1;
    int nq = min(a.q_count ? a.q_count[b] : a.T, 16 * NQT);
    float mrun[NQT], lrun[NQT];
    f32x4 oacc[NQT][4];
    attn_wave<NQT, VBLK, true, !VBLK>(a, b, h, 0, nq, 0, 1, L.vs[wave], mrun, lrun, oacc);
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
  const bf16* hb = L.hb;
  auto getB = [&](int t, int k) { return *reinterpret_cast<const bf16x8*>(hb + (t * 16 + lq) * pitch + k); };
  auto slice = [&](auto ic) {
    constexpr int I = decltype(ic)::value;
    const int vb = w + kRsWorkers * I;
    if (vb >= P::nvb) return;
    f32x4 acc[2];
    rs_slice_mma<PER, d, TWO, I>(pre, W, vb, k0, getB, acc);
    const int n0 = vb * 16;
    const float* hown = L.hown + I * kSkRows * 16;
    sk_reduce(acc, L.red, R, [&](int m, int nl, float v) {
      st_coh(xs_out + (size_t)m * d + n0 + nl, v + (float)bias[n0 + nl] + hown[m * 16 + nl]);
    });
    __syncthreads();
  };
  static_assert(P::NSL <= 2, "residual slices per workgroup");
  slice(std::integral_constant<int, 0>{});
  if constexpr (P::NSL > 1) slice(std::integral_constant<int, 1>{});
}

// xs_out = hidden(resid) + hid W2^T + bias; hid bf16 [R][F] written by the previous phase
template <int PER, int FS, bool TWO>
__device__ __forceinline__ void rs_ffn2(const SkLds<PER>& L, const SkSrc& resid, int R, const bf16* hid,
                                        const bf16* __restrict__ W, const bf16* __restrict__ bias, float* xs_out,
                                        int w, const bf16x8 (&pre)[kRsPre]) {
  constexpr int d = 64 * PER, F = 128 * FS, S1 = FS < kSkW ? FS : kSkW, nvb = d / 16;
  constexpr int NSL = (nvb + kRsWorkers - 1) / kRsWorkers;
  const int wave = threadIdx.x >> 6, lq = threadIdx.x & 15, g = (threadIdx.x & 63) >> 4;
  const int k0 = wave * (F / 4);
  if (w >= nvb) return;
  const int vb1 = w + kRsWorkers;
  // first-tile activations of this wave's k range (the same for every slice)
  bf16x8 hf[S1];
  {
    const bf16* hp = hid + (size_t)min(lq, R - 1) * F + k0 + 8 * g;
#pragma unroll
    for (int u = 0; u < S1; ++u) hf[u] = ld_coh16(hp + u * 32);
  }
  sk_hidden<PER, true>(resid, R, TWO ? 32 : 16, L.hb, L.hown, w * 16, false, vb1 < nvb ? vb1 * 16 : -64);
  auto getB = [&](int t, int k) { return ld_coh16(hid + (size_t)min(t * 16 + lq, R - 1) * F + k); };
  __syncthreads();
  auto slice = [&](auto ic) {
    constexpr int I = decltype(ic)::value;
    const int vb = w + kRsWorkers * I;
    if (vb >= nvb) return;
    const int n0 = vb * 16;
    f32x4 acc[2];
    sk_zero(acc);
    bf16x8 wf[S1];
    if constexpr (I > 0) sk_wload<S1>(W, F, n0, d, k0, wf);
#pragma unroll
    for (int u = 0; u < S1; ++u) {
      const bf16x8 wv = (I == 0) ? pre[u] : wf[u];
      acc[0] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(wv, hf[u], acc[0], 0, 0, 0);
      if (TWO) acc[1] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(wv, getB(1, k0 + u * 32 + 8 * g), acc[1], 0, 0, 0);
    }
    mfma_settle(acc[0], acc[1]);
    sk_mma_tail<FS, TWO>(W, F, n0, d, k0, getB, acc);
    mfma_settle(acc[0], acc[1]);
    const float* hown = L.hown + I * kSkRows * 16;
    sk_reduce(acc, L.red, R, [&](int m, int nl, float v) {
      st_coh(xs_out + (size_t)m * d + n0 + nl, v + (float)bias[n0 + nl] + hown[m * 16 + nl]);
    });
    __syncthreads();
  };
  static_assert(NSL <= 2, "residual slices per workgroup");
  slice(std::integral_constant<int, 0>{});
  if constexpr (NSL > 1) slice(std::integral_constant<int, 1>{});
}

// ---- vocabulary helpers --------------------------------------------------------------------
// Workgroups beyond the first kRsWorkers take no part in the decoder phases: each requests its
// vocabulary tiles (and the embedding rows of the drafts) at once, sleeps until workgroup 0
// publishes the launch number in the done flag, then needs only the final hidden state.
constexpr int kRsHeld = 3;   // tiles a helper holds in registers

template <int PER, bool TWO>
__device__ __forceinline__ void rs_vocab_helper(const SkLds<PER>& L, const RsArgs& A, float* zd_lds, int* flag) {
  constexpr int d = 64 * PER, pitch = d + kSkPad, steps = d / 32, S1 = steps < kSkW ? steps : kSkW;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, lq = lane & 15, g = lane >> 4;
  const int h = blockIdx.x - kRsWorkers, NH = gridDim.x - kRsWorkers;
  const int V = A.V, R = A.R, n_tiles = (V + 63) / 64;
  const bf16* __restrict__ E = A.E;
  unsigned* err = A.bar + 16;
  unsigned* done = A.bar + kRsFlagPitch * (1 + h);   // this helper's own wake-up word
  // requests that depend on nothing the pass computes
  bf16x8 wf[kRsHeld][S1];
#pragma unroll
  for (int i = 0; i < kRsHeld; ++i)
    if (h + NH * i < n_tiles) sk_wload<S1>(E, d, (h + NH * i) * 64 + wave * 16, V, 0, wf[i]);
  const int drow = wave * 16 + lq;                       // waves 0, 1: the draft this lane's row scores
  const int dtok = (wave < 2 && drow < R) ? A.row_draft[drow] : -1;
  const bool dhas = dtok >= 0 && dtok < V;
  bf16x8 dw[S1];
  {
    const bf16* wp = E + (size_t)(dhas ? dtok : 0) * d + 8 * g;
#pragma unroll
    for (int u = 0; u < S1; ++u) dw[u] = *reinterpret_cast<const bf16x8*>(wp + u * 32);
  }
  // bounded wait for the decoder
  if (threadIdx.x == 0) {
    unsigned spins = 0;
    int bad = 0;
    while (__hip_atomic_load(done, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) != (unsigned)A.seq) {
      if (++spins > kRsSpinMax || __hip_atomic_load(err, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) != 0u) {
        __hip_atomic_store(err, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        bad = 1;
        break;
      }
      __builtin_amdgcn_s_sleep(64);
    }
    *flag = bad;
  }
  __syncthreads();
  if (*flag) return;
  // final hidden state = LayerNorm 3 of the last layer's residual sum
  const RsLayer& Ly = A.layers[A.n_layers - 1];
  const SkSrc src{2, ((A.n_layers - 1) & 1) ? A.xs1 : A.xs0, Ly.ln3g, Ly.ln3b, nullptr, nullptr, nullptr, nullptr};
  sk_hidden<PER, true>(src, R, TWO ? 32 : 16, L.hb, L.hown, -64, true);
  __syncthreads();
  const bf16* hb = L.hb;
  // draft logits: same instruction and k order as the tiles below (bit-identical elements)
  if (wave < 2) {
    f32x4 acc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int u = 0; u < S1; ++u)
      acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(dw[u], *reinterpret_cast<const bf16x8*>(hb + drow * pitch + u * 32 + 8 * g), acc, 0, 0, 0);
    if constexpr (steps > S1) {
      const bf16* wp = E + (size_t)(dhas ? dtok : 0) * d + 8 * g;
#pragma unroll 8
      for (int u = S1; u < steps; ++u)
        acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(*reinterpret_cast<const bf16x8*>(wp + u * 32),
                                                      *reinterpret_cast<const bf16x8*>(hb + drow * pitch + u * 32 + 8 * g), acc, 0, 0, 0);
    }
    mfma_settle(acc);
    if (g == (lq >> 2) && drow < R) {
      float v = 0.f;
#pragma unroll
      for (int r = 0; r < 4; ++r) if (r == (lq & 3)) v = acc[r];
      v = dhas ? v : kNegInf;
      zd_lds[drow] = v;
      if (h == 0) A.zd[drow] = v;
    }
  }
  __syncthreads();
  float zd[2];
#pragma unroll
  for (int t = 0; t < 2; ++t) zd[t] = (t * 16 + lq < R) ? zd_lds[t * 16 + lq] : kNegInf;
  auto getB = [&](int t, int k) { return *reinterpret_cast<const bf16x8*>(hb + (t * 16 + lq) * pitch + k); };
  auto tile = [&](int vb, const bf16x8 (&w16)[S1]) {
    const int n0 = vb * 64 + wave * 16;
    f32x4 acc[2];
    sk_zero(acc);
    sk_mma<S1, TWO>(w16, 0, getB, acc);
    sk_mma_tail<steps, TWO>(E, d, n0, V, 0, getB, acc);
    mfma_settle(acc[0], acc[1]);
    sk_vocab_tile(acc, n0, V, R, zd, L.red, A.part, n_tiles, vb, A.logits);
    __syncthreads();
  };
#pragma unroll
  for (int i = 0; i < kRsHeld; ++i)
    if (h + NH * i < n_tiles) tile(h + NH * i, wf[i]);
  for (int vb = h + NH * kRsHeld; vb < n_tiles; vb += NH) {   // more tiles than a helper holds
    bf16x8 w16[S1];
    sk_wload<S1>(E, d, vb * 64 + wave * 16, V, 0, w16);
    tile(vb, w16);
  }
}

// ---- the kernel ----------------------------------------------------------------------------
template <int PER, int FS, bool TWO>
__global__ __launch_bounds__(kSkThreads) void rs_verify_kernel(RsArgs A) {
  extern __shared__ __attribute__((aligned(16))) char sk_smem[];
  SkLds<PER> L(sk_smem);
  float* zd_lds = reinterpret_cast<float*>(sk_smem + SkLds<PER>::kBytes);   // [32]
  int* flag = reinterpret_cast<int*>(zd_lds + kSkRows);
  constexpr int d = 64 * PER, F = 128 * FS;
  const int w = blockIdx.x, R = A.R;
  unsigned* err = A.bar + 16;
  if (__hip_atomic_load(err, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) != 0u) return;   // sticky error: do nothing
  if (w >= kRsWorkers) {
    rs_vocab_helper<PER, TWO>(L, A, zd_lds, flag);
    return;
  }
  RsState bar{A.bar + A.parity, err, 0u, flag};
  if (w == 0 && threadIdx.x == 0) __hip_atomic_store(A.bar + (1 - A.parity), 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);

  SkSrc cur{0, nullptr, nullptr, nullptr, A.row_tok, A.row_pos, A.E, A.pe};
  float* freeb = A.xs0;
  float* other = A.xs1;
  auto produced = [&](const bf16* g, const bf16* b) {
    cur = SkSrc{2, freeb, g, b, nullptr, nullptr, nullptr, nullptr};
    float* t = freeb; freeb = other; other = t;
  };
  bf16x8 pre[kRsPre];
  rs_prefetch_proj<PER, 3 * d>(pre, A.layers[0].wqkv, w);
  for (int l = 0; l < A.n_layers; ++l) {
    const RsLayer& Ly = A.layers[l];
    bf16* kc = A.kc + A.kv_layer * l;
    bf16* vc = A.vc + A.kv_layer * l;
    // QKV + append
    rs_project<PER, 3 * d, TWO>(L, cur, R, Ly.wqkv, w, pre, [&](int m, int n, float v) {
      v += (float)Ly.bqkv[n];
      const int part = n / d, c = n - part * d;
      if (part == 0) { st_coh(A.q + (size_t)m * d + c, (bf16)v); return; }
      const int b = A.row_b[m];
      if (b < 0) return;
      bf16* cache = (part == 1) ? kc : vc;
      st_coh(cache + (((size_t)b * A.H + (c >> 6)) * A.Lcap + A.row_pos[m]) * kHeadDim + (c & 63), (bf16)v);
    });
    rs_arrive(bar);
    rs_prefetch_proj<PER, d>(pre, Ly.wo, w);
    if (!rs_wait(bar)) return;
    // self-attention + O
    AttnArgs a{};
    a.q = A.q; a.q_b = (long)A.T * d; a.q_row = d;
    a.k = kc; a.k_b = (long)A.H * A.Lcap * 64; a.k_h = (long)A.Lcap * 64; a.k_row = 64;
    a.v = vc; a.v_b = a.k_b; a.v_h = a.k_h; a.v_row = 64; a.v_blocked = 0;
    a.q_count = A.seq_rows; a.lim_row = A.row_lim; a.lim_seq = nullptr;
    a.T = A.T; a.H = A.H; a.B = A.B; a.key_split = 0; a.cap = A.Lcap;
    rs_attn_o<PER, false, TWO>(L, cur, R, a, Ly.wo, Ly.bo, freeb, w, pre);
    produced(Ly.ln1g, Ly.ln1b);
    rs_arrive(bar);
    rs_prefetch_proj<PER, d>(pre, Ly.cwq, w);
    if (!rs_wait(bar)) return;
    // cross-attention Q
    rs_project<PER, d, TWO>(L, cur, R, Ly.cwq, w, pre, [&](int m, int n, float v) {
      st_coh(A.q + (size_t)m * d + n, (bf16)(v + (float)Ly.cbq[n]));
    });
    rs_arrive(bar);
    rs_prefetch_proj<PER, d>(pre, Ly.cwo, w);
    if (!rs_wait(bar)) return;
    // cross-attention + O
    a.k = A.xk + A.xkv_layer * l; a.k_b = (long)A.H * A.Scap * 64; a.k_h = (long)A.Scap * 64;
    a.v = A.xv + A.xkv_layer * l; a.v_b = a.k_b; a.v_h = a.k_h; a.v_blocked = 1;
    a.lim_row = nullptr; a.lim_seq = A.src_len; a.cap = A.Scap;
    rs_attn_o<PER, true, TWO>(L, cur, R, a, Ly.cwo, Ly.cbo, freeb, w, pre);
    produced(Ly.ln2g, Ly.ln2b);
    rs_arrive(bar);
    rs_prefetch_proj<PER, F>(pre, Ly.w1, w);
    if (!rs_wait(bar)) return;
    // FFN1
    rs_project<PER, F, TWO>(L, cur, R, Ly.w1, w, pre, [&](int m, int n, float v) {
      st_coh(A.hid + (size_t)m * F + n, (bf16)fmaxf(v + (float)Ly.b1[n], 0.f));
    });
    rs_arrive(bar);
    rs_prefetch_ffn2<PER, FS>(pre, Ly.w2, w);
    if (!rs_wait(bar)) return;
    // FFN2
    rs_ffn2<PER, FS, TWO>(L, cur, R, A.hid, Ly.w2, Ly.b2, freeb, w, pre);
    produced(Ly.ln3g, Ly.ln3b);
    rs_arrive(bar);
    if (l + 1 < A.n_layers) rs_prefetch_proj<PER, 3 * d>(pre, A.layers[l + 1].wqkv, w);
    if (!rs_wait(bar)) return;
  }
  // the final residual sum is visible everywhere: wake the vocabulary helpers, each through a
  // word of its own (one hot word polled by every helper would saturate its memory channel)
  const int helpers = (int)gridDim.x - kRsWorkers;
  for (int h = w * kSkThreads + threadIdx.x; h < helpers; h += kRsWorkers * kSkThreads)
    __hip_atomic_store(A.bar + kRsFlagPitch * (1 + h), (unsigned)A.seq, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

// ---- launcher ------------------------------------------------------------------------------
#define RS_DISPATCH(d, CALL)                          \
  switch ((d) / 64) {                                 \
    case 2: { constexpr int PER = 2; CALL; } break;   \
    case 8: { constexpr int PER = 8; CALL; } break;   \
    case 16: { constexpr int PER = 16; CALL; } break; \
    default: return hipErrorInvalidValue;             \
  }
#define RS_FFN(F, CALL)                               \
  switch ((F) / 128) {                                \
    case 2: { constexpr int FS = 2; CALL; } break;    \
    case 16: { constexpr int FS = 16; CALL; } break;  \
    case 32: { constexpr int FS = 32; CALL; } break;  \
    default: return hipErrorInvalidValue;             \
  }
#define RS_ROWS(R, CALL)                                        \
  if ((R) > 16) { constexpr bool TWO = true; CALL; }            \
  else { constexpr bool TWO = false; CALL; }

template <int PER, int FS, bool TWO>
static hipError_t rs_launch(hipStream_t st, const RsArgs& A) {
  constexpr int lds = (int)SkLds<PER>::kBytes + kSkRows * 4 + 16;
  static bool ready = false;   // attribute of this instantiation, set once per process
  if (!ready) {
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(rs_verify_kernel<PER, FS, TWO>),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, lds);
    if (e != hipSuccess) return e;
    ready = true;
  }
  const int n_tiles = (A.V + 63) / 64;
  const int helpers = n_tiles < kRsHelpers ? n_tiles : kRsHelpers;
  hipLaunchKernelGGL((rs_verify_kernel<PER, FS, TWO>), dim3(kRsWorkers + helpers), dim3(kSkThreads), lds, st, A);
  return hipGetLastError();
}

hipError_t resident_verify(hipStream_t st, const RsArgs& A, int d, int F) {
  if (A.R < 1 || A.R > kSkRows || A.T > kSkRows || A.seq == 0 || !skinny_supported(d, F)) return hipErrorInvalidValue;
  RS_DISPATCH(d, RS_FFN(F, RS_ROWS(A.R, return (rs_launch<PER, FS, TWO>(st, A)))));
  return hipErrorInvalidValue;
}

}  // namespace sd
