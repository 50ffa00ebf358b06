// Small kernels around the GEMMs: embedding, LayerNorm, row assembly, the acceptance test
// (paper Sec. 3.2, Eq. 8-10), commit (Sec. 2, Eq. 3) and state / cache marshalling.
#include "common.h"
#include "kernels.h"

namespace sd {

static inline dim3 blocks_for(long n, int t) { return dim3((unsigned)((n + t - 1) / t)); }

// ----------------------------------------------------------------------------- positions
// PE(p, 2i) = sin(p / 10000^(2i/d)), PE(p, 2i+1) = cos(same), evaluated in fp64.
__global__ void pos_table_kernel(float* pe, int n_pos, int d) {
  long idx = (long)blockIdx.x * blockDim.x + threadIdx.x;
  if (idx >= (long)n_pos * d) return;
  int p = (int)(idx / d), c = (int)(idx % d);
  int i = c >> 1;
  double ang = (double)p / pow(10000.0, 2.0 * (double)i / (double)d);
  pe[idx] = (float)((c & 1) ? cos(ang) : sin(ang));
}
hipError_t build_pos_table(hipStream_t st, float* pe, int n_pos, int d) {
  long n = (long)n_pos * d;
  hipLaunchKernelGGL(pos_table_kernel, blocks_for(n, 256), dim3(256), 0, st, pe, n_pos, d);
  return hipGetLastError();
}

// ----------------------------------------------------------------------------- embedding
// x[r] = E[tok[r]] * sqrt(d) + PE[pos[r]]  (fp32) and its bf16 copy
// One block per row, 8 columns per thread and step (d % 64 == 0).
__device__ __forceinline__ void embed_row(const bf16* __restrict__ e, const float* __restrict__ p,
                                          float* __restrict__ xr, bf16* __restrict__ xbr, int d, float scale) {
  for (int c = threadIdx.x * 8; c < d; c += blockDim.x * 8) {
    const bf16x8 ev = *reinterpret_cast<const bf16x8*>(e + c);
    const f32x4 p0 = *reinterpret_cast<const f32x4*>(p + c), p1 = *reinterpret_cast<const f32x4*>(p + c + 4);
    f32x4 v0, v1;
    bf16x8 o;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      v0[i] = (float)ev[i] * scale + p0[i];
      v1[i] = (float)ev[4 + i] * scale + p1[i];
      o[i] = (bf16)v0[i];
      o[4 + i] = (bf16)v1[i];
    }
    *reinterpret_cast<f32x4*>(xr + c) = v0;
    *reinterpret_cast<f32x4*>(xr + c + 4) = v1;
    *reinterpret_cast<bf16x8*>(xbr + c) = o;
  }
}
__global__ __launch_bounds__(128) void embed_kernel(const int* __restrict__ tok, const int* __restrict__ pos,
                                                    const bf16* __restrict__ E, const float* __restrict__ pe,
                                                    float* __restrict__ x, bf16* __restrict__ xb, int R, int d,
                                                    float scale) {
  const int r = blockIdx.x;
  if (r >= R) return;
  embed_row(E + (size_t)tok[r] * d, pe + (size_t)pos[r] * d, x + (size_t)r * d, xb + (size_t)r * d, d, scale);
}
hipError_t embed_rows(hipStream_t st, const int* tok, const int* pos, const bf16* E,
                      const float* pe, float* x, bf16* xb, int R, int d) {
  if (R <= 0) return hipSuccess;
  hipLaunchKernelGGL(embed_kernel, dim3(R), dim3(128), 0, st, tok, pos, E, pe, x, xb, R, d,
                     sqrtf((float)d));
  return hipGetLastError();
}

// ----------------------------------------------------------------------------- LayerNorm
// One wave per row; mean and biased variance as two reductions over registers; eps 1e-5.
// All loads of a row are issued before the first use (PER is a compile-time count), so a
// row costs one memory round trip, not one per element.
template <int PER>   // d = 64 * PER
__global__ __launch_bounds__(256) void ln_kernel(float* __restrict__ x, const bf16* __restrict__ g,
                                                 const bf16* __restrict__ bta, bf16* __restrict__ xb,
                                                 int R, const int* __restrict__ m_real) {
  constexpr int d = 64 * PER;
  const int lane = threadIdx.x & 63;
  const int r = blockIdx.x * 4 + (threadIdx.x >> 6);
  if (r >= R || (m_real && r >= *m_real)) return;
  float* xr = x + (size_t)r * d;
  float v[PER], gg[PER], bb[PER];
#pragma unroll
  for (int i = 0; i < PER; ++i) v[i] = xr[i * 64 + lane];
#pragma unroll
  for (int i = 0; i < PER; ++i) { gg[i] = (float)g[i * 64 + lane]; bb[i] = (float)bta[i * 64 + lane]; }
  float s = 0.f;
#pragma unroll
  for (int i = 0; i < PER; ++i) s += v[i];
  const float mean = wave_sum(s) / (float)d;
  float q = 0.f;
#pragma unroll
  for (int i = 0; i < PER; ++i) { float t = v[i] - mean; q += t * t; }
  const float rstd = fast_rsqrt(wave_sum(q) / (float)d + 1e-5f);
#pragma unroll
  for (int i = 0; i < PER; ++i) {
    const int c = i * 64 + lane;
    const float y = (v[i] - mean) * rstd * gg[i] + bb[i];
    xr[c] = y;
    xb[(size_t)r * d + c] = (bf16)y;
  }
}
// The same on the drafter's mask-slot rows only: output row o = b*k + s is the LayerNorm of row
// b*T + new_rows[b] + s of x, written (bf16 only) to the dense [B*k][d] operand of the
// vocabulary kernel.
template <int PER>
__global__ __launch_bounds__(256) void ln_slots_kernel(const float* __restrict__ x, const bf16* __restrict__ g,
                                                       const bf16* __restrict__ bta, bf16* __restrict__ dst,
                                                       const int* __restrict__ new_rows,
                                                       const int* __restrict__ row_start, int B, int T, int k) {
  constexpr int d = 64 * PER;
  const int lane = threadIdx.x & 63;
  const int o = blockIdx.x * 4 + (threadIdx.x >> 6);
  if (o >= B * k) return;
  const int b = o / k, sl = o - b * k;
  const float* xr = x + (size_t)((row_start ? row_start[b] : b * T) + new_rows[b] + sl) * d;
  float v[PER], gg[PER], bb[PER];
#pragma unroll
  for (int i = 0; i < PER; ++i) v[i] = xr[i * 64 + lane];
#pragma unroll
  for (int i = 0; i < PER; ++i) { gg[i] = (float)g[i * 64 + lane]; bb[i] = (float)bta[i * 64 + lane]; }
  float s = 0.f;
#pragma unroll
  for (int i = 0; i < PER; ++i) s += v[i];
  const float mean = wave_sum(s) / (float)d;
  float q = 0.f;
#pragma unroll
  for (int i = 0; i < PER; ++i) { float t = v[i] - mean; q += t * t; }
  const float rstd = fast_rsqrt(wave_sum(q) / (float)d + 1e-5f);
#pragma unroll
  for (int i = 0; i < PER; ++i)
    dst[(size_t)o * d + i * 64 + lane] = (bf16)((v[i] - mean) * rstd * gg[i] + bb[i]);
}
template <int PER>
static hipError_t ln_slots_launch(hipStream_t st, const float* x, const bf16* g, const bf16* b, bf16* dst,
                                  const int* new_rows, const int* row_start, int B, int T, int k) {
  hipLaunchKernelGGL(ln_slots_kernel<PER>, dim3((B * k + 3) / 4), dim3(256), 0, st, x, g, b, dst, new_rows, row_start,
                     B, T, k);
  return hipGetLastError();
}
hipError_t layer_norm_slots(hipStream_t st, const float* x, const bf16* g, const bf16* b, bf16* dst,
                            const int* new_rows, const int* row_start, int B, int T, int k, int d) {
  if (B <= 0 || k <= 0) return hipSuccess;
  switch (d / 64) {
#define SD_LN_CASE(P) case P: return ln_slots_launch<P>(st, x, g, b, dst, new_rows, row_start, B, T, k);
    SD_LN_CASE(1) SD_LN_CASE(2) SD_LN_CASE(3) SD_LN_CASE(4) SD_LN_CASE(5) SD_LN_CASE(6) SD_LN_CASE(7) SD_LN_CASE(8)
    SD_LN_CASE(9) SD_LN_CASE(10) SD_LN_CASE(11) SD_LN_CASE(12) SD_LN_CASE(13) SD_LN_CASE(14) SD_LN_CASE(15)
    SD_LN_CASE(16) SD_LN_CASE(17) SD_LN_CASE(18) SD_LN_CASE(19) SD_LN_CASE(20) SD_LN_CASE(21) SD_LN_CASE(22)
    SD_LN_CASE(23) SD_LN_CASE(24) SD_LN_CASE(25) SD_LN_CASE(26) SD_LN_CASE(27) SD_LN_CASE(28) SD_LN_CASE(29)
    SD_LN_CASE(30) SD_LN_CASE(31) SD_LN_CASE(32)
#undef SD_LN_CASE
    default: return hipErrorInvalidValue;
  }
}

template <int PER>
static hipError_t ln_launch(hipStream_t st, float* x, const bf16* g, const bf16* b, bf16* xb, int R, const int* m_real) {
  hipLaunchKernelGGL(ln_kernel<PER>, dim3((R + 3) / 4), dim3(256), 0, st, x, g, b, xb, R, m_real);
  return hipGetLastError();
}
hipError_t layer_norm(hipStream_t st, float* x, const bf16* g, const bf16* b, bf16* xb, int R, int d, const int* m_real) {
  if (R <= 0) return hipSuccess;
  switch (d / 64) {   // d = 64 * heads, heads <= 32
#define SD_LN_CASE(P) case P: return ln_launch<P>(st, x, g, b, xb, R, m_real);
    SD_LN_CASE(1) SD_LN_CASE(2) SD_LN_CASE(3) SD_LN_CASE(4) SD_LN_CASE(5) SD_LN_CASE(6) SD_LN_CASE(7) SD_LN_CASE(8)
    SD_LN_CASE(9) SD_LN_CASE(10) SD_LN_CASE(11) SD_LN_CASE(12) SD_LN_CASE(13) SD_LN_CASE(14) SD_LN_CASE(15)
    SD_LN_CASE(16) SD_LN_CASE(17) SD_LN_CASE(18) SD_LN_CASE(19) SD_LN_CASE(20) SD_LN_CASE(21) SD_LN_CASE(22)
    SD_LN_CASE(23) SD_LN_CASE(24) SD_LN_CASE(25) SD_LN_CASE(26) SD_LN_CASE(27) SD_LN_CASE(28) SD_LN_CASE(29)
    SD_LN_CASE(30) SD_LN_CASE(31) SD_LN_CASE(32)
#undef SD_LN_CASE
    default: return hipErrorInvalidValue;
  }
}

__global__ void fill_i32_kernel(int* p, int v, long n) {
  long i = (long)blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n) p[i] = v;
}
hipError_t fill_i32(hipStream_t st, int* p, int v, long n) {
  if (n <= 0) return hipSuccess;
  hipLaunchKernelGGL(fill_i32_kernel, blocks_for(n, 256), dim3(256), 0, st, p, v, n);
  return hipGetLastError();
}

// ----------------------------------------------------------------------------- verify rows
// Row i of sequence b: token u_j (i = 0) or draft i (i >= 1) at position j + i; it may look
// at keys [0, j + i + 1) and it scores draft i + 1 (none on the last row).
__global__ void assemble_verify_kernel(SeqState s, RowMap rm, const int* __restrict__ draft, int B, int k, int V) {
  int idx = blockIdx.x * blockDim.x + threadIdx.x;
  int T = k + 1;
  if (idx >= B * T) return;
  int b = idx / T, i = idx - b * T;
  int j = s.len[b];
  int tok = (i == 0) ? s.tokens[(size_t)b * s.tok_pitch + j] : draft[b * k + i - 1];
  rm.row_b[idx] = b;
  rm.row_pos[idx] = j + i;
  rm.row_tok[idx] = min(max(tok, 0), V - 1);   // ids index the embedding table
  rm.row_lim[idx] = j + i + 1;
  rm.row_draft[idx] = (i < k) ? draft[b * k + i] : -1;
  if (i < k) s.last_draft[b * s.k_max + i] = draft[b * k + i];
  if (i == 0) rm.seq_rows[b] = T;
}
hipError_t assemble_verify(hipStream_t st, const SeqState& s, const RowMap& rm, const int* draft, int B, int k, int V) {
  hipLaunchKernelGGL(assemble_verify_kernel, blocks_for((long)B * (k + 1), 128), dim3(128), 0, st, s, rm, draft, B, k, V);
  return hipGetLastError();
}
// The same, one block per row, followed by the row's embedding (embed_rows).
__global__ __launch_bounds__(128) void assemble_embed_verify_kernel(SeqState s, RowMap rm,
                                                                    const int* __restrict__ draft, int B, int k, int V,
                                                                    const bf16* __restrict__ E,
                                                                    const float* __restrict__ pe,
                                                                    float* __restrict__ x, bf16* __restrict__ xb, int d,
                                                                    float scale) {
  const int idx = blockIdx.x, T = k + 1;
  const int b = idx / T, i = idx - b * T;
  const int j = s.len[b];
  int tok = (i == 0) ? s.tokens[(size_t)b * s.tok_pitch + j] : draft[b * k + i - 1];
  tok = min(max(tok, 0), V - 1);
  if (threadIdx.x == 0) {
    rm.row_b[idx] = b;
    rm.row_pos[idx] = j + i;
    rm.row_tok[idx] = tok;
    rm.row_lim[idx] = j + i + 1;
    rm.row_draft[idx] = (i < k) ? draft[b * k + i] : -1;
    if (i < k) s.last_draft[b * s.k_max + i] = draft[b * k + i];
    if (i == 0) rm.seq_rows[b] = T;
  }
  embed_row(E + (size_t)tok * d, pe + (size_t)(j + i) * d, x + (size_t)idx * d, xb + (size_t)idx * d, d, scale);
}
hipError_t assemble_embed_verify(hipStream_t st, const SeqState& s, const RowMap& rm, const int* draft, int B, int k,
                                 int V, const bf16* E, const float* pe, float* x, bf16* xb, int d) {
  if (B <= 0) return hipSuccess;
  hipLaunchKernelGGL(assemble_embed_verify_kernel, dim3(B * (k + 1)), dim3(128), 0, st, s, rm, draft, B, k, V, E, pe,
                     x, xb, d, sqrtf((float)d));
  return hipGetLastError();
}

// ----------------------------------------------------------------------------- prefill / draft rows
// Each sequence owns up to T row slots of the pass.
// Prefill (n_mask = 0): the next up to T uncached stream tokens, causal.
// Draft (Sec. 3.1.3, Eq. 7): the uncached stream tokens (causal) followed by n_mask [MASK]
// slots; slot s sits at the position of the token it predicts and attends to the whole stream
// and to all slots.  The slots' keys/values land beyond the valid cache length and are dead
// after the pass.  new_rows[b] = stream rows of this pass (the amount `cached` advances by).
// One block per row: the row's bookkeeping, then its embedding (embed_rows).  PACKED: the rows
// of the sequences follow each other without padding; a block finds its sequence's first row as
// the sum of the row counts of the sequences before it (each thread derives some of them from the
// state, as the block does for its own), and blocks beyond their sequence's rows do nothing.
struct StreamRows {
  int c0, n, rows;
  bool masks;
};
__device__ __forceinline__ StreamRows stream_rows(const SeqState& s, int role, int b, int T, int n_mask) {
  StreamRows r;
  r.c0 = s.cached[role][b];
  const int target = s.len[b] + (role == 1 ? 1 : 0);       // drafter also ingests the pending token
  r.n = max(0, min(target - r.c0, T - n_mask));
  r.masks = n_mask > 0 && r.c0 + r.n == target;             // slots only once the stream is ingested
  r.rows = r.n + (r.masks ? n_mask : 0);
  return r;
}
template <bool PACKED>
__global__ __launch_bounds__(128) void assemble_embed_stream_kernel(SeqState s, RowMap rm, int role, int B, int T,
                                                                    int n_mask, int mask_id, int pad_id, int V,
                                                                    int* __restrict__ new_rows,
                                                                    const bf16* __restrict__ E,
                                                                    const float* __restrict__ pe,
                                                                    float* __restrict__ x, bf16* __restrict__ xb, int d,
                                                                    float scale) {
  __shared__ int wsum[2];
  const int b = blockIdx.x / T, i = blockIdx.x - b * T;
  const StreamRows me = stream_rows(s, role, b, T, n_mask);
  int first = b * T;
  if (PACKED) {
    int part = 0;
    for (int o = threadIdx.x; o < b; o += 128) part += stream_rows(s, role, o, T, n_mask).rows;
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) part += __shfl_xor(part, off, 64);
    if ((threadIdx.x & 63) == 0) wsum[threadIdx.x >> 6] = part;
    __syncthreads();
    first = wsum[0] + wsum[1];
  }
  if (threadIdx.x == 0 && i == 0) {
    rm.seq_rows[b] = me.rows;
    new_rows[b] = me.n;
    if (PACKED) {
      rm.row_start[b] = first;
      if (b == B - 1) rm.row_start[B] = first + me.rows;
    }
  }
  if (PACKED && i >= me.rows) return;
  const int r = first + i;
  int rb = -1, pos = 0, tok = pad_id, lim = 0;
  if (i < me.n) {
    rb = b; pos = me.c0 + i; tok = min(max(s.tokens[(size_t)b * s.tok_pitch + me.c0 + i], 0), V - 1); lim = me.c0 + i + 1;
  } else if (me.masks && i < me.n + n_mask) {
    rb = b; pos = me.c0 + i; tok = mask_id; lim = me.c0 + me.n + n_mask;
  }
  if (threadIdx.x == 0) {
    rm.row_b[r] = rb; rm.row_pos[r] = pos; rm.row_tok[r] = tok; rm.row_lim[r] = lim; rm.row_draft[r] = -1;
  }
  embed_row(E + (size_t)tok * d, pe + (size_t)pos * d, x + (size_t)r * d, xb + (size_t)r * d, d, scale);
}
hipError_t assemble_embed_stream(hipStream_t st, const SeqState& s, const RowMap& rm, int role, int B, int T,
                                 int n_mask, int mask_id, int pad_id, int V, int* new_rows, const bf16* E,
                                 const float* pe, float* x, bf16* xb, int d, bool packed) {
  if (B <= 0 || T <= 0) return hipSuccess;
  if (packed)
    hipLaunchKernelGGL(assemble_embed_stream_kernel<true>, dim3(B * T), dim3(128), 0, st, s, rm, role, B, T, n_mask,
                       mask_id, pad_id, V, new_rows, E, pe, x, xb, d, sqrtf((float)d));
  else
    hipLaunchKernelGGL(assemble_embed_stream_kernel<false>, dim3(B * T), dim3(128), 0, st, s, rm, role, B, T, n_mask,
                       mask_id, pad_id, V, new_rows, E, pe, x, xb, d, sqrtf((float)d));
  return hipGetLastError();
}

__global__ void advance_cached_kernel(SeqState s, int role, const int* __restrict__ new_rows, int B) {
  const int b = blockIdx.x * blockDim.x + threadIdx.x;
  if (b < B) s.cached[role][b] += new_rows[b];
}
hipError_t advance_cached(hipStream_t st, const SeqState& s, int role, const int* new_rows, int B) {
  hipLaunchKernelGGL(advance_cached_kernel, blocks_for(B, 64), dim3(64), 0, st, s, role, new_rows, B);
  return hipGetLastError();
}

// dense [B*k][d] copy of the mask-slot rows (row b*T + new_rows[b] + s) for the vocabulary kernel
__global__ void gather_slots_kernel(const bf16* __restrict__ xb, bf16* __restrict__ dst,
                                    const int* __restrict__ new_rows, const int* __restrict__ row_start, int B, int T,
                                    int k, int d) {
  const int o = blockIdx.x;              // b*k + s
  const int b = o / k, sl = o - b * k;
  const int first = row_start ? row_start[b] : b * T;
  const uint4* src = reinterpret_cast<const uint4*>(xb + (size_t)(first + new_rows[b] + sl) * d);
  uint4* out = reinterpret_cast<uint4*>(dst + (size_t)o * d);
  for (int c = threadIdx.x; c < d / 8; c += blockDim.x) out[c] = src[c];
}
hipError_t gather_slots(hipStream_t st, const bf16* xb, bf16* dst, const int* new_rows, const int* row_start, int B,
                        int T, int k, int d) {
  hipLaunchKernelGGL(gather_slots_kernel, dim3(B * k), dim3(64), 0, st, xb, dst, new_rows, row_start, B, T, k, d);
  return hipGetLastError();
}

// encoder rows: row b*S + s feeds src[b][s] (clamped into the vocabulary) at position s
__global__ void encoder_rows_kernel(const int* __restrict__ src, int* __restrict__ tok, int* __restrict__ pos,
                                    long n, int S, int V) {
  const long i = (long)blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= n) return;
  tok[i] = min(max(src[i], 0), V - 1);
  pos[i] = (int)(i % S);
}
hipError_t encoder_rows(hipStream_t st, const int* src, int* tok, int* pos, int B, int S, int V) {
  const long n = (long)B * S;
  hipLaunchKernelGGL(encoder_rows_kernel, blocks_for(n, 256), dim3(256), 0, st, src, tok, pos, n, S, V);
  return hipGetLastError();
}

// The same without the padding: sequence b owns rows row_start[b] .. row_start[b] + src_len[b] - 1 (a
// running sum, sources in batch order), n_rows[0] = their number.  Rows beyond it (up to B * S) get a
// valid token, position 0 and sequence -1: whatever is computed on them is never stored anywhere else.
__global__ __launch_bounds__(1024) void encoder_pack_scan_kernel(const int* __restrict__ src_len, int B, int S,
                                                                 int* __restrict__ row_start, int* __restrict__ n_rows) {
  __shared__ int part[1024];
  const int per = (B + 1023) / 1024, b0 = threadIdx.x * per;
  int sum = 0;
  for (int i = 0; i < per; ++i)
    if (b0 + i < B) sum += min(max(src_len[b0 + i], 0), S);
  part[threadIdx.x] = sum;
  __syncthreads();
  if (threadIdx.x == 0) {
    int run = 0;
    for (int t = 0; t < 1024; ++t) { const int v = part[t]; part[t] = run; run += v; }
    row_start[B] = run;
    n_rows[0] = run;
  }
  __syncthreads();
  int run = part[threadIdx.x];
  for (int i = 0; i < per; ++i)
    if (b0 + i < B) { row_start[b0 + i] = run; run += min(max(src_len[b0 + i], 0), S); }
}
__global__ void encoder_pack_rows_kernel(const int* __restrict__ src, const int* __restrict__ src_len,
                                         const int* __restrict__ row_start, int* __restrict__ tok,
                                         int* __restrict__ pos, int* __restrict__ row_b, long n, int B, int S, int V) {
  const long i = (long)blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= n) return;
  const int b = (int)(i / S), s = (int)(i - (long)b * S);
  if (s < min(max(src_len[b], 0), S)) {
    const int r = row_start[b] + s;
    tok[r] = min(max(src[i], 0), V - 1);
    pos[r] = s;
    row_b[r] = b;
  }
  if (i >= row_start[B]) { tok[i] = 0; pos[i] = 0; row_b[i] = -1; }   // (the rows no sequence owns)
}
hipError_t encoder_rows_packed(hipStream_t st, const int* src, const int* src_len, int* tok, int* pos, int* row_b,
                               int* row_start, int* n_rows, int B, int S, int V) {
  const long n = (long)B * S;
  hipLaunchKernelGGL(encoder_pack_scan_kernel, dim3(1), dim3(1024), 0, st, src_len, B, S, row_start, n_rows);
  hipLaunchKernelGGL(encoder_pack_rows_kernel, blocks_for(n, 256), dim3(256), 0, st, src, src_len, row_start, tok, pos,
                     row_b, n, B, S, V);
  return hipGetLastError();
}

// dst [B][S][d] <- the packed rows of every sequence, zeros beyond its length
__global__ void unpack_rows_kernel(const bf16* __restrict__ src, const int* __restrict__ row_start,
                                   const int* __restrict__ src_len, bf16* __restrict__ dst, long n8, int S, int d) {
  const long i = (long)blockIdx.x * blockDim.x + threadIdx.x;   // one 16-byte piece
  if (i >= n8) return;
  const int per = d / 8;
  const long row = i / per;
  const int c = (int)(i - row * per) * 8;
  const int b = (int)(row / S), s = (int)(row - (long)b * S);
  bf16x8 v;
#pragma unroll
  for (int e = 0; e < 8; ++e) v[e] = (bf16)0.f;
  if (s < min(max(src_len[b], 0), S)) v = *reinterpret_cast<const bf16x8*>(src + (size_t)(row_start[b] + s) * d + c);
  *reinterpret_cast<bf16x8*>(dst + (size_t)row * d + c) = v;
}
hipError_t unpack_rows(hipStream_t st, const bf16* src, const int* row_start, const int* src_len, bf16* dst, int B,
                       int S, int d) {
  const long n8 = (long)B * S * (d / 8);
  if (n8 <= 0) return hipSuccess;
  hipLaunchKernelGGL(unpack_rows_kernel, blocks_for(n8, 256), dim3(256), 0, st, src, row_start, src_len, dst, n8, S, d);
  return hipGetLastError();
}

// ----------------------------------------------------------------------------- acceptance
// Stage 1, one wave per row: merge the per-tile partials of the vocabulary kernel into
//   m = max logit, arg-max = lowest column among maxima, LSE, and the number of logits that
//   are strictly larger than the logit z_d of the draft this row scores.
struct RowMerge {
  float m, lse;
  int arg, cnt;
};
__device__ __forceinline__ RowMerge merge_row(const float* __restrict__ pr, int n_tiles, int lane) {
  constexpr int kHeld = 8;   // records per lane kept in registers: one pass over memory up to 512 tiles
  const bool held = n_tiles <= 64 * kHeld;
  f32x4 rec[kHeld];
  float m = kNegInf;
  int am = 0x7fffffff, cnt = 0;
  if (held) {
#pragma unroll
    for (int i = 0; i < kHeld; ++i)   // (clamped, so that no load sits behind a lane's own branch)
      rec[i] = *reinterpret_cast<const f32x4*>(pr + (size_t)min(lane + 64 * i, n_tiles - 1) * kPartF);
#pragma unroll
    for (int i = 0; i < kHeld; ++i) {
      if (lane + 64 * i < n_tiles) {
        const float tm = rec[i][0];
        const int ti = __float_as_int(rec[i][1]);
        if (tm > m || (tm == m && ti < am)) { m = tm; am = ti; }
        cnt += __float_as_int(rec[i][3]);
      }
    }
  } else {
    for (int t = lane; t < n_tiles; t += 64) {
      const f32x4 p = *reinterpret_cast<const f32x4*>(pr + (size_t)t * kPartF);
      const float tm = p[0];
      const int ti = __float_as_int(p[1]);
      if (tm > m || (tm == m && ti < am)) { m = tm; am = ti; }
      cnt += __float_as_int(p[3]);
    }
  }
  const float gm = wave_max(m);
  int cand = (m == gm) ? am : 0x7fffffff;
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) {
    cand = min(cand, __shfl_xor(cand, o, 64));
    cnt += __shfl_xor(cnt, o, 64);
  }
  float se = 0.f;
  if (held) {
#pragma unroll
    for (int i = 0; i < kHeld; ++i)
      if (lane + 64 * i < n_tiles) se += rec[i][2] * __expf(rec[i][0] - gm);
  } else {
    for (int t = lane; t < n_tiles; t += 64) {
      const f32x4 p = *reinterpret_cast<const f32x4*>(pr + (size_t)t * kPartF);
      se += p[2] * __expf(p[0] - gm);
    }
  }
  se = wave_sum(se);
  return RowMerge{gm, gm + __logf(se), cand, cnt};
}
__device__ __forceinline__ void store_row_stats(float* rs, const RowMerge& r, float zd) {
  *reinterpret_cast<f32x4*>(rs) = f32x4{r.m, (float)r.arg, r.lse, zd};
  *reinterpret_cast<f32x4*>(rs + 4) = f32x4{(float)r.cnt, 0.f, 0.f, 0.f};
}

// Stage 2, per sequence (paper Sec. 3.2).  With z_d the draft's logit on its row:
// Eq. 8:  log P(draft) >= log P(beta-th ranked)   <=>  #{v : z_v > z_d} < beta
// Eq. 9:  log P(top-1) - log P(draft) <= tau      <=>  m - z_d <= tau
// (log-softmax subtracts the same LSE from every logit of the row; a draft tied with the
// beta-th score passes, as ">=" says).  a = number of leading rows that pass; next = arg-max
// of row a.
//
// Both stages in one launch: a block per sequence, its 16 waves merge the k + 1 <= 32 rows (two
// rounds at most), then one thread scans them.
constexpr int kMergeWaves = 16;
__global__ __launch_bounds__(64 * kMergeWaves) void merge_accept_kernel(const float* __restrict__ part,
                                                           const float* __restrict__ zd_row, int n_tiles,
                                                           float* __restrict__ row_stats, SeqState s, int k,
                                                           int beta, float tau, int pad_id,
                                                           int* __restrict__ accept_len,
                                                           int* __restrict__ next_token,
                                                           const unsigned* __restrict__ fail) {
  __shared__ float sm[32], szd[32];
  __shared__ int sarg[32], scnt[32];
  const int b = blockIdx.x, lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int T = k + 1;
  for (int i = wave; i < T; i += kMergeWaves) {
    const int r = b * T + i;
    const RowMerge res = merge_row(part + (size_t)r * n_tiles * kPartF, n_tiles, lane);
    if (lane == 0) {
      const float zd = zd_row[r];
      store_row_stats(row_stats + (size_t)r * kRowStats, res, zd);
      sm[i] = res.m; szd[i] = zd; sarg[i] = res.arg; scnt[i] = res.cnt;
    }
  }
  __syncthreads();
  if (threadIdx.x != 0) return;
  if (fail && *fail) { accept_len[b] = -1; next_token[b] = pad_id; return; }
  // keys/values of u_0..u_{j-1} must be cached: a cache loaded short of the stream (and not
  // completed by a prefill) would have let this pass attend to rows that were never written
  if (s.cached[0][b] < s.len[b] && !s.finished[b]) { accept_len[b] = -1; next_token[b] = pad_id; return; }
  int a = 0;
  for (; a < k; ++a)
    if (!(scnt[a] < beta && sm[a] - szd[a] <= tau)) break;
  const bool fin = s.finished[b] != 0;
  accept_len[b] = fin ? 0 : a;
  next_token[b] = fin ? pad_id : sarg[a];
  if (!fin) {   // rows whose tau test was decided by a margin of at most 1e-2 (up to the bifurcation row)
    int near = 0;
    for (int i = 0; i <= a && i < k; ++i) near += fabsf(tau - (sm[i] - szd[i])) <= 1e-2f ? 1 : 0;
    if (near) atomicAdd(&s.scratch[3], near);
  }
}
hipError_t merge_accept(hipStream_t st, const float* part, const float* zd_row, int n_tiles, float* row_stats,
                        const SeqState& s, int B, int k, int beta, float tau, int pad_id, int* accept_len,
                        int* next_token, const unsigned* fail) {
  if (B <= 0) return hipSuccess;
  if (k + 1 > 32) return hipErrorInvalidValue;
  hipLaunchKernelGGL(merge_accept_kernel, dim3(B), dim3(64 * kMergeWaves), 0, st, part, zd_row, n_tiles, row_stats, s, k, beta,
                     tau, pad_id, accept_len, next_token, fail);
  return hipGetLastError();
}

// Drafter: merge the slot rows, draft[b][s] = arg-max of slot row b*k + s (pad for finished
// sequences); the first B blocks also advance the drafter's cached length by the stream rows
// this pass ingested.
__global__ __launch_bounds__(64) void merge_drafts_kernel(const float* __restrict__ part, int n_tiles,
                                                          float* __restrict__ row_stats, SeqState s, int B, int k,
                                                          int pad_id, const int* __restrict__ new_rows,
                                                          const int* __restrict__ seq_rows,
                                                          int* __restrict__ draft) {
  const int o = blockIdx.x, lane = threadIdx.x;
  const RowMerge res = merge_row(part + (size_t)o * n_tiles * kPartF, n_tiles, lane);
  if (lane != 0) return;
  store_row_stats(row_stats + (size_t)o * kRowStats, res, kNegInf);
  // a sequence whose uncached stream did not fit into this pass got no mask slots (its rows of
  // the pass were all stream rows): what sits at its slot rows belongs to another sequence
  const int b = o / k;
  const bool has_slots = seq_rows[b] - new_rows[b] == k;
  draft[o] = (s.finished[b] || !has_slots) ? pad_id : res.arg;
  if (o < B) s.cached[1][o] += new_rows[o];
}
hipError_t merge_drafts(hipStream_t st, const float* part, int n_tiles, float* row_stats, const SeqState& s, int B,
                        int k, int pad_id, const int* new_rows, const int* seq_rows, int* draft) {
  if (B <= 0 || k <= 0) return hipSuccess;
  hipLaunchKernelGGL(merge_drafts_kernel, dim3(B * k), dim3(64), 0, st, part, n_tiles, row_stats, s, B, k, pad_id,
                     new_rows, seq_rows, draft);
  return hipGetLastError();
}

// ----------------------------------------------------------------------------- head-based drafting
// Input rows of the drafting heads (Sec. 2 "Draft": FFN heads on the target model's last hidden
// state): for sequence b the verifier's final hidden state at the bifurcation row a_b of the
// latest pass (the row whose arg-max is next_token).  x holds the pass's rows [B*T][d], already
// normalised (g == null) or as the last residual sum still to be normalised with (g, beta).
// Written as bf16 [B][d] (GEMM operand) and, replicated k times, as fp32 [B*k][d] (the residual
// each head adds to).  One wave per sequence.
template <int PER>
__global__ __launch_bounds__(256) void head_rows_kernel(const float* __restrict__ x, const bf16* __restrict__ g,
                                                        const bf16* __restrict__ beta,
                                                        const int* __restrict__ accept_len, int B, int T, int k,
                                                        bf16* __restrict__ rows, float* __restrict__ rep) {
  constexpr int d = 64 * PER;
  const int lane = threadIdx.x & 63;
  const int b = blockIdx.x * 4 + (threadIdx.x >> 6);
  if (b >= B) return;
  const int a = min(max(accept_len[b], 0), T - 1);
  const float* xr = x + ((size_t)b * T + a) * d;
  float v[PER];
#pragma unroll
  for (int i = 0; i < PER; ++i) v[i] = xr[i * 64 + lane];
  if (g) {
    float s = 0.f;
#pragma unroll
    for (int i = 0; i < PER; ++i) s += v[i];
    const float mean = wave_sum(s) / (float)d;
    float q = 0.f;
#pragma unroll
    for (int i = 0; i < PER; ++i) { float t = v[i] - mean; q += t * t; }
    const float rstd = fast_rsqrt(wave_sum(q) / (float)d + 1e-5f);
#pragma unroll
    for (int i = 0; i < PER; ++i) v[i] = (v[i] - mean) * rstd * (float)g[i * 64 + lane] + (float)beta[i * 64 + lane];
  }
#pragma unroll
  for (int i = 0; i < PER; ++i) {
    const int c = i * 64 + lane;
    rows[(size_t)b * d + c] = (bf16)v[i];
    for (int h = 0; h < k; ++h) rep[((size_t)b * k + h) * d + c] = v[i];
  }
}
template <int PER>
static hipError_t head_rows_launch(hipStream_t st, const float* x, const bf16* g, const bf16* beta, const int* accept_len,
                                   int B, int T, int k, bf16* rows, float* rep) {
  hipLaunchKernelGGL(head_rows_kernel<PER>, dim3((B + 3) / 4), dim3(256), 0, st, x, g, beta, accept_len, B, T, k, rows, rep);
  return hipGetLastError();
}
hipError_t head_rows(hipStream_t st, const float* x, const bf16* g, const bf16* beta, const int* accept_len, int B, int T,
                     int k, int d, bf16* rows, float* rep) {
  if (B <= 0 || k <= 0) return hipSuccess;
  switch (d / 64) {
#define SD_LN_CASE(P) case P: return head_rows_launch<P>(st, x, g, beta, accept_len, B, T, k, rows, rep);
    SD_LN_CASE(1) SD_LN_CASE(2) SD_LN_CASE(3) SD_LN_CASE(4) SD_LN_CASE(5) SD_LN_CASE(6) SD_LN_CASE(7) SD_LN_CASE(8)
    SD_LN_CASE(9) SD_LN_CASE(10) SD_LN_CASE(11) SD_LN_CASE(12) SD_LN_CASE(13) SD_LN_CASE(14) SD_LN_CASE(15)
    SD_LN_CASE(16) SD_LN_CASE(17) SD_LN_CASE(18) SD_LN_CASE(19) SD_LN_CASE(20) SD_LN_CASE(21) SD_LN_CASE(22)
    SD_LN_CASE(23) SD_LN_CASE(24) SD_LN_CASE(25) SD_LN_CASE(26) SD_LN_CASE(27) SD_LN_CASE(28) SD_LN_CASE(29)
    SD_LN_CASE(30) SD_LN_CASE(31) SD_LN_CASE(32)
#undef SD_LN_CASE
    default: return hipErrorInvalidValue;
  }
}

__global__ void f32_to_bf16_kernel(const float* __restrict__ src, bf16* __restrict__ dst, long n) {
  const long i = ((long)blockIdx.x * blockDim.x + threadIdx.x) * 4;
  if (i >= n) return;   // n % 4 == 0
  const f32x4 v = *reinterpret_cast<const f32x4*>(src + i);
  bf16x4 o;
#pragma unroll
  for (int e = 0; e < 4; ++e) o[e] = (bf16)v[e];
  *reinterpret_cast<bf16x4*>(dst + i) = o;
}
hipError_t f32_to_bf16(hipStream_t st, const float* src, bf16* dst, long n) {
  if (n <= 0) return hipSuccess;
  hipLaunchKernelGGL(f32_to_bf16_kernel, blocks_for(n / 4, 256), dim3(256), 0, st, src, dst, n);
  return hipGetLastError();
}

// draft[b][i] = arg-max of head row b*k + i (pad for finished sequences and for sequences whose
// verification reported a failure)
__global__ __launch_bounds__(64) void merge_head_drafts_kernel(const float* __restrict__ part, int n_tiles,
                                                               float* __restrict__ row_stats, SeqState s,
                                                               const int* __restrict__ accept_len, int k, int pad_id,
                                                               int* __restrict__ draft) {
  const int o = blockIdx.x, lane = threadIdx.x;
  const RowMerge res = merge_row(part + (size_t)o * n_tiles * kPartF, n_tiles, lane);
  if (lane != 0) return;
  store_row_stats(row_stats + (size_t)o * kRowStats, res, kNegInf);
  const int b = o / k;
  draft[o] = (s.finished[b] || accept_len[b] < 0) ? pad_id : res.arg;
}
hipError_t merge_head_drafts(hipStream_t st, const float* part, int n_tiles, float* row_stats, const SeqState& s,
                             const int* accept_len, int B, int k, int pad_id, int* draft) {
  if (B <= 0 || k <= 0) return hipSuccess;
  hipLaunchKernelGGL(merge_head_drafts_kernel, dim3(B * k), dim3(64), 0, st, part, n_tiles, row_stats, s, accept_len, k,
                     pad_id, draft);
  return hipGetLastError();
}

// ----------------------------------------------------------------------------- commit
// Eq. 3: the iteration's output is the accepted drafts followed by the verifier's token; a
// sequence stops after its first EOS or when it reaches its cap.  j advances by the number
// of tokens appended: exactly that many of this pass's cache rows become valid.
__global__ void commit_kernel(SeqState s, const int* __restrict__ accept_len, const int* __restrict__ next_token,
                              int B, int k, int eos_id, int* n_active) {
  __shared__ int active, tokens;
  if (threadIdx.x == 0) { active = 0; tokens = 0; }
  __syncthreads();
  // the counters are read now and written at the end: their round trip runs under the sequences'
  int c_commits = 0, c_tokens = 0;
  if (threadIdx.x == 0) { c_commits = s.scratch[0]; c_tokens = s.scratch[1]; }
  int mine = 0, added = 0;
  for (int b = threadIdx.x; b < B; b += blockDim.x) {
    // one memory round trip per sequence: the scalars and, whatever they turn out to be, every token
    // that may be appended (k_max <= 31 drafts are stored per sequence)
    const int fin0 = s.finished[b], a0 = accept_len[b], j0 = s.len[b], cap = s.cap[b], nt = next_token[b];
    int t[32];
#pragma unroll
    for (int i = 0; i < 31; ++i) t[i] = (i < k) ? s.last_draft[b * s.k_max + i] : 0;
    t[31] = 0;
    if (fin0) continue;
    if (a0 < 0) { ++mine; continue; }   // verification reported a failure: nothing to commit
    const int a = min(a0, k);   // k of the pass whose drafts are stored: entries beyond it are stale
    int j = j0;
    int* u = s.tokens + (size_t)b * s.tok_pitch;
    int fin = 0;
#pragma unroll
    for (int i = 0; i < 32; ++i) {
      if (i <= a && !fin) {
        if (j >= cap) {
          fin = 1;
        } else {
          const int tok = (i < a) ? t[i] : nt;
          u[++j] = tok;
          if (tok == eos_id || j >= cap) fin = 1;
        }
      }
    }
    added += j - j0;
    s.len[b] = j;
    s.cached[0][b] = j;   // the verifier's rows of the kept tokens are now valid cache
    s.finished[b] = fin;
    if (!fin) ++mine;
  }
  if (mine) atomicAdd(&active, mine);
  if (added) atomicAdd(&tokens, added);
  __syncthreads();
  if (threadIdx.x == 0) {
    if (n_active) *n_active = active;
    s.scratch[0] = c_commits + 1;        // commits
    s.scratch[1] = c_tokens + tokens;    // tokens appended
    s.scratch[2] = B - active;  // finished sequences
  }
}
hipError_t commit_rows(hipStream_t st, const SeqState& s, const int* accept_len, const int* next_token, int B,
                       int k, int eos_id, int* n_active) {
  hipLaunchKernelGGL(commit_kernel, dim3(1), dim3(256), 0, st, s, accept_len, next_token, B, min(k, s.k_max), eos_id,
                     n_active);
  return hipGetLastError();
}

// ----------------------------------------------------------------------------- state
__global__ void begin_kernel(SeqState s, int B, int max_new, int max_tgt, int bos_id) {
  int b = blockIdx.x * blockDim.x + threadIdx.x;
  if (b < 8) s.scratch[b] = 0;   // counters: commits, tokens appended, finished, near-threshold rows
  if (b >= B) return;
  s.tokens[(size_t)b * s.tok_pitch] = bos_id;
  s.len[b] = 0;
  s.start[b] = 0;
  s.cap[b] = min(max_new, max_tgt);
  s.finished[b] = (max_new <= 0);
  s.cached[0][b] = 0;
  s.cached[1][b] = 0;
}
hipError_t begin_state(hipStream_t st, const SeqState& s, int B, int max_new, int max_tgt, int bos_id) {
  hipLaunchKernelGGL(begin_kernel, blocks_for(B, 128), dim3(128), 0, st, s, B, max_new, max_tgt, bos_id);
  return hipGetLastError();
}

__global__ void set_stream_kernel(SeqState s, const int* __restrict__ tokens, const int* __restrict__ len, int B,
                                  int L_max, int max_new, int max_tgt) {
  int b = blockIdx.x;
  if (b >= B) return;
  int j = min(max(len[b], 0), L_max);
  for (int i = threadIdx.x; i <= j; i += blockDim.x)
    s.tokens[(size_t)b * s.tok_pitch + i] = tokens[(size_t)b * (L_max + 1) + i];
  if (threadIdx.x == 0) {
    s.len[b] = j;
    s.start[b] = j;
    const int cap = j + min(max_new, max(max_tgt - j, 0));   // (max_new may be huge: no j + max_new)
    s.cap[b] = cap;
    s.finished[b] = (j >= cap);
    s.cached[0][b] = 0;
    s.cached[1][b] = 0;
  }
}
hipError_t set_stream(hipStream_t st, const SeqState& s, const int* tokens, const int* len, int B, int L_max,
                      int max_new, int max_tgt) {
  hipLaunchKernelGGL(set_stream_kernel, dim3(B), dim3(64), 0, st, s, tokens, len, B, L_max, max_new, max_tgt);
  return hipGetLastError();
}

// Rollback to given lengths: nothing moves, rows beyond the new j are dead.
__global__ void rewind_kernel(SeqState s, const int* __restrict__ len, int B) {
  int b = blockIdx.x * blockDim.x + threadIdx.x;
  if (b >= B) return;
  int j = s.len[b];
  int jn = min(j, max(len[b], 0));
  if (jn < j) {
    s.len[b] = jn;
    s.start[b] = min(s.start[b], jn);
    s.cached[0][b] = min(s.cached[0][b], jn);
    s.cached[1][b] = min(s.cached[1][b], jn + 1);
    s.finished[b] = (jn >= s.cap[b]);
  }
}
hipError_t rewind_state(hipStream_t st, const SeqState& s, const int* len, int B) {
  hipLaunchKernelGGL(rewind_kernel, blocks_for(B, 128), dim3(128), 0, st, s, len, B);
  return hipGetLastError();
}

__global__ void copy_i32_kernel(int* dst, const int* src, int n) {
  int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n) dst[i] = src[i];
}
__global__ void clamp_copy_i32_kernel(int* dst, const int* src, int n, int lo, int hi) {
  int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n) dst[i] = min(max(src[i], lo), hi);
}
hipError_t set_src_len(hipStream_t st, const SeqState& s, const int* src_len, int B, int S_max) {
  hipLaunchKernelGGL(clamp_copy_i32_kernel, blocks_for(B, 128), dim3(128), 0, st, s.src_len, src_len, B, 1, S_max);
  return hipGetLastError();
}
hipError_t set_cached(hipStream_t st, const SeqState& s, int role, const int* n, int B, int hi) {
  hipLaunchKernelGGL(clamp_copy_i32_kernel, blocks_for(B, 128), dim3(128), 0, st, s.cached[role], n, B, 0, hi);
  return hipGetLastError();
}

__global__ void get_output_kernel(SeqState s, int* __restrict__ tokens, int out_cap, int* __restrict__ out_len,
                                  int* __restrict__ finished, int B, int pad_id) {
  int b = blockIdx.x;
  if (b >= B) return;
  int st0 = s.start[b], n = s.len[b] - st0;
  for (int i = threadIdx.x; i < out_cap; i += blockDim.x)
    tokens[(size_t)b * out_cap + i] = (i < n) ? s.tokens[(size_t)b * s.tok_pitch + st0 + 1 + i] : pad_id;
  if (threadIdx.x == 0) {
    out_len[b] = n;
    if (finished) finished[b] = s.finished[b];
  }
}
hipError_t get_output(hipStream_t st, const SeqState& s, int* tokens, int out_cap, int* out_len, int* finished,
                      int B, int pad_id) {
  hipLaunchKernelGGL(get_output_kernel, dim3(B), dim3(64), 0, st, s, tokens, out_cap, out_len, finished, B, pad_id);
  return hipGetLastError();
}

// ----------------------------------------------------------------------------- cache layout
// flat [B][L][H*64]  <->  key cache [B][H][Lcap][64] (16-byte chunks) or transposed value
// cache (element-wise; only used to load / inspect caches)
__global__ void cache_flat_kernel(bf16* cache, bf16* flat, int B, int H, int Lcap, int L, int to_flat) {
  long idx = (long)blockIdx.x * blockDim.x + threadIdx.x;
  long n = (long)B * L * H * 8;
  if (idx >= n) return;
  int ch = (int)(idx & 7);
  long t = idx >> 3;
  int h = (int)(t % H); t /= H;
  int l = (int)(t % L);
  int b = (int)(t / L);
  uint4* c = reinterpret_cast<uint4*>(cache + (((size_t)b * H + h) * Lcap + l) * kHeadDim + ch * 8);
  uint4* f = reinterpret_cast<uint4*>(flat + (((size_t)b * L + l) * H + h) * kHeadDim + ch * 8);
  if (to_flat) *f = *c; else *c = *f;
}
__global__ void cache_flat_t_kernel(bf16* cache, bf16* flat, int B, int H, int Lcap, int L, int to_flat) {
  long idx = (long)blockIdx.x * blockDim.x + threadIdx.x;
  long n = (long)B * L * H * kHeadDim;
  if (idx >= n) return;
  int e = (int)(idx & 63);
  long t = idx >> 6;
  int h = (int)(t % H); t /= H;
  int l = (int)(t % L);
  int b = (int)(t / L);
  bf16* c = cache + ((size_t)b * H + h) * Lcap * kHeadDim + vt_off(l, e);
  bf16* f = flat + (((size_t)b * L + l) * H + h) * kHeadDim + e;
  if (to_flat) *f = *c; else *c = *f;
}
static hipError_t cache_flat(hipStream_t st, bf16* cache, bf16* flat, int B, int H, int Lcap, int L, bool tr, int to_flat) {
  if ((long)B * L <= 0) return hipSuccess;
  if (tr) {
    long n = (long)B * L * H * kHeadDim;
    hipLaunchKernelGGL(cache_flat_t_kernel, blocks_for(n, 256), dim3(256), 0, st, cache, flat, B, H, Lcap, L, to_flat);
  } else {
    long n = (long)B * L * H * 8;
    hipLaunchKernelGGL(cache_flat_kernel, blocks_for(n, 256), dim3(256), 0, st, cache, flat, B, H, Lcap, L, to_flat);
  }
  return hipGetLastError();
}
hipError_t cache_from_flat(hipStream_t st, bf16* cache, const bf16* flat, int B, int H, int Lcap, int L, bool tr) {
  return cache_flat(st, cache, const_cast<bf16*>(flat), B, H, Lcap, L, tr, 0);
}
hipError_t cache_to_flat(hipStream_t st, const bf16* cache, bf16* flat, int B, int H, int Lcap, int L, bool tr) {
  return cache_flat(st, const_cast<bf16*>(cache), flat, B, H, Lcap, L, tr, 1);
}

// ---- FP8 E4M3 weight storage (1-4-3, bias 7, largest value 448, no infinities) ----------------
// Nearest code of |x|, ties to the even mantissa, saturating at 448 (0x7e).
__device__ __forceinline__ unsigned e4m3_code(float x) {
  const unsigned sign = (__float_as_uint(x) >> 24) & 0x80u;
  const float a = fabsf(x);
  unsigned code;
  if (a >= 448.f) {
    code = 0x7eu;
  } else if (a < 0x1p-6f) {
    const unsigned q = (unsigned)rintf(a * 512.f);   // subnormal grid: multiples of 2^-9
    code = q >= 8u ? 0x08u : q;
  } else {
    const unsigned bits = __float_as_uint(a);
    int E = (int)(bits >> 23) - 127;
    unsigned m = (bits >> 20) & 7u;
    const unsigned rem = bits & 0xfffffu;
    if (rem > 0x80000u || (rem == 0x80000u && (m & 1u))) ++m;
    if (m == 8u) { m = 0u; ++E; }
    code = min(((unsigned)(E + 7) << 3) | m, 0x7eu);
  }
  return code | sign;
}
__global__ __launch_bounds__(256) void quantize_rows_kernel(const bf16* __restrict__ w, int K,
                                                            unsigned char* __restrict__ codes,
                                                            float* __restrict__ scale) {
  __shared__ float red[4];
  const bf16* row = w + (size_t)blockIdx.x * K;
  float amax = 0.f;
  for (int k = threadIdx.x * 8; k < K; k += 256 * 8) {
    const bf16x8 v = *reinterpret_cast<const bf16x8*>(row + k);
#pragma unroll
    for (int i = 0; i < 8; ++i) amax = fmaxf(amax, fabsf((float)v[i]));
  }
  amax = wave_max(amax);
  if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = amax;
  __syncthreads();
  amax = fmaxf(fmaxf(red[0], red[1]), fmaxf(red[2], red[3]));
  const float s = amax > 0.f ? __fdiv_rn(amax, 448.f) : 1.f;
  if (threadIdx.x == 0) scale[blockIdx.x] = s;
  for (int k = threadIdx.x * 8; k < K; k += 256 * 8) {
    const bf16x8 v = *reinterpret_cast<const bf16x8*>(row + k);
    unsigned lo = 0, hi = 0;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      lo |= e4m3_code(__fdiv_rn((float)v[i], s)) << (8 * i);
      hi |= e4m3_code(__fdiv_rn((float)v[4 + i], s)) << (8 * i);
    }
    *reinterpret_cast<uint2*>(codes + (size_t)blockIdx.x * K + k) = make_uint2(lo, hi);
  }
}
// One wave per block of 8 keys.  Keys: lane = (row lane/8, dims 8*(lane%8) .. +7).  Values (key-blocked:
// element (key r, dim e) of the block at e*8 + r): lane = dim e, its 8 elements are the 8 keys.
__global__ __launch_bounds__(256) void quantize_cross_kv_kernel(const bf16* __restrict__ xk, const bf16* __restrict__ xv,
                                                                long n_blocks, unsigned char* __restrict__ k8,
                                                                unsigned char* __restrict__ v8, float* __restrict__ ksc,
                                                                float* __restrict__ vsc) {
  const long blk = (long)blockIdx.x * 4 + (threadIdx.x >> 6);
  if (blk >= n_blocks) return;
  const int lane = threadIdx.x & 63;
  const long off = blk * 512 + lane * 8;
  {
    const bf16x8 v = *reinterpret_cast<const bf16x8*>(xk + off);
    float amax = 0.f;
#pragma unroll
    for (int i = 0; i < 8; ++i) amax = fmaxf(amax, fabsf((float)v[i]));
    amax = fmaxf(amax, __shfl_xor(amax, 1, 64));
    amax = fmaxf(amax, __shfl_xor(amax, 2, 64));
    amax = fmaxf(amax, __shfl_xor(amax, 4, 64));
    const float s = amax > 0.f ? __fdiv_rn(amax, 448.f) : 1.f;
    unsigned lo = 0, hi = 0;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      lo |= e4m3_code(__fdiv_rn((float)v[i], s)) << (8 * i);
      hi |= e4m3_code(__fdiv_rn((float)v[4 + i], s)) << (8 * i);
    }
    *reinterpret_cast<uint2*>(k8 + off) = make_uint2(lo, hi);
    if ((lane & 7) == 0) ksc[blk * 8 + (lane >> 3)] = s;
  }
  {
    const bf16x8 v = *reinterpret_cast<const bf16x8*>(xv + off);
    unsigned lo = 0, hi = 0;
#pragma unroll
    for (int r = 0; r < 8; ++r) {
      const float amax = wave_max(fabsf((float)v[r]));
      const float s = amax > 0.f ? __fdiv_rn(amax, 448.f) : 1.f;
      const unsigned code = e4m3_code(__fdiv_rn((float)v[r], s));
      if (r < 4) lo |= code << (8 * r); else hi |= code << (8 * (r - 4));
      if (lane == r) vsc[blk * 8 + r] = s;
    }
    *reinterpret_cast<uint2*>(v8 + off) = make_uint2(lo, hi);
  }
}
hipError_t quantize_cross_kv(hipStream_t st, const bf16* xk, const bf16* xv, long rows, unsigned char* k8,
                             unsigned char* v8, float* ksc, float* vsc) {
  if (rows <= 0) return hipSuccess;
  if (rows % 8 != 0 || rows / 8 > 0x7fffffffL * 4) return hipErrorInvalidValue;
  const long n_blocks = rows / 8;
  hipLaunchKernelGGL(quantize_cross_kv_kernel, dim3((unsigned)((n_blocks + 3) / 4)), dim3(256), 0, st, xk, xv, n_blocks, k8,
                     v8, ksc, vsc);
  return hipGetLastError();
}

hipError_t quantize_rows_e4m3(hipStream_t st, const bf16* w, int N, int K, unsigned char* codes, float* scale) {
  if (N <= 0) return hipSuccess;
  if (K <= 0 || K % 8 != 0) return hipErrorInvalidValue;
  hipLaunchKernelGGL(quantize_rows_kernel, dim3(N), dim3(256), 0, st, w, K, codes, scale);
  return hipGetLastError();
}

}  // namespace sd
