// Host-side launchers of the gfx950 kernels.  Plain pointers and sizes; every function
// enqueues on `st` and returns the launch status.  Shapes are validated by the callers in
// api.hip before anything is launched.
#pragma once
#include <hip/hip_runtime.h>
#include <hip/hip_ext.h>
#include <stdint.h>

namespace sd {

typedef __bf16 bf16;

// Row bookkeeping of one decoder pass.  Row r belongs to sequence row_b[r] (-1 = padding
// row: computed but never stored into a cache), sits at stream position row_pos[r], feeds
// token row_tok[r], may attend to self-attention keys [0, row_lim[r]) and scores draft token
// row_draft[r] (-1 = none).  Rows of sequence b are b*T .. b*T + seq_rows[b] - 1, or, in a
// packed pass, row_start[b] .. row_start[b] + seq_rows[b] - 1 with row_start the running sum of
// seq_rows (row_start[B] = number of rows of the pass): no padding rows between sequences.
struct RowMap {
  int* row_b;
  int* row_pos;
  int* row_tok;
  int* row_lim;
  int* row_draft;
  int* seq_rows;
  int* row_start;   // [B + 1]
};

// ---- gemm.hip: C = A W^T (+bias) with different epilogues; A [M,K] bf16, W [N,K] bf16 ----
// m_real (device, nullable, here and below): number of leading rows that hold data; row tiles at or beyond it
// are skipped, rows beyond it neither read nor stored (M stays the upper bound the grid is sized for).
// out fp32 [M,ldo] = A W^T + bias + resid (resid may alias out, may be null)
hipError_t gemm_f32(hipStream_t st, const bf16* A, int lda, const bf16* W, int M, int N, int K,
                    const bf16* bias, const float* resid, float* out, int ldo, const int* m_real = nullptr);
// out bf16 [M,ldo] = act(A W^T + bias)
hipError_t gemm_bf16(hipStream_t st, const bf16* A, int lda, const bf16* W, int M, int N, int K,
                     const bf16* bias, bf16* out, int ldo, bool relu, const int* m_real = nullptr);
// Self-attention projection of decoder rows, N = 3d: q -> q_out [M,d]; k, v of row r ->
// caches [B][H][Lcap][64] at sequence row_b[r], position row_pos[r] (the KV append).
hipError_t gemm_qkv_append(hipStream_t st, const bf16* A, const bf16* W, int M, int d, int K,
                           const bf16* bias, bf16* q_out, bf16* kc, bf16* vc, const int* row_b,
                           const int* row_pos, int H, int Lcap, const int* m_real = nullptr);
// Cross-attention keys/values of the encoder memory, N = 2d: memory row m -> sequence b, source position s ->
// xk [B][H][Scap][64], xv key-blocked [B][H][Scap/8][64][8].  Padded rows (row_b null): m = b*S + s; packed
// rows: b = row_b[m] (negative: a row no sequence owns, dropped), s = row_s[m].
hipError_t gemm_cross_kv(hipStream_t st, const bf16* A, const bf16* W, int M, int d, int K,
                         const bf16* bias, bf16* xk, bf16* xv, int S, int H, int Scap, const int* row_b = nullptr,
                         const int* row_s = nullptr, const int* m_real = nullptr);

// Encoder self-attention projection, N = 3d, rows as above: q -> q_out [M,d] (row m), keys ->
// ek [B][H][Scap][64], values -> ev key-blocked [B][H][Scap/8][64][8].
hipError_t gemm_enc_qkv(hipStream_t st, const bf16* A, const bf16* W, int M, int d, int K,
                        const bf16* bias, bf16* q_out, bf16* ek, bf16* ev, int S, int H, int Scap,
                        const int* row_b = nullptr, const int* row_s = nullptr, const int* m_real = nullptr);

// ---- LayerNorm folded into the GEMM around it (post-LN blocks) ----
// y = residual sum of a sub-layer, LN(y) = (y - mean) * rstd * g + beta.  The GEMM that forms y
// also writes bf16(y * g) and, per row and 64-column chunk, the pair {sum, squared deviations
// from the chunk mean} ("chunk pairs", fp32 [M][pitch][2], pitch = d/64 rounded up to even); the GEMMs that consume LN(y) multiply
// bf16(y * g) and finish with rstd * (acc - mean * cs) + bf.
struct LnFold {          // per consuming weight matrix W [N,d] with bias b, for one LayerNorm (g, beta)
  const float* cs;       // [N]  sum_k g[k] W[n][k]
  const float* bf;       // [N]  b[n] + sum_k beta[k] W[n][k]
};
hipError_t ln_fold(hipStream_t st, const bf16* W, const bf16* g, const bf16* beta, const bf16* b, int N, int K,
                   const LnFold& out);
// The column vectors of one producing GEMM, fp32 [3][d] in one piece: gain of the LayerNorm
// pending on the residual (1 when g_prev is null), its shift (0 when null) + the GEMM's bias,
// gain of the LayerNorm that follows.
hipError_t ln_sum_vecs(hipStream_t st, const bf16* bias, const bf16* g_prev, const bf16* b_prev, const bf16* g_next,
                       int d, float* out);
// x [M,d] += A W^T + bias, where the residual already in x is LN_prev(x) if has_prev (chunk pairs of
// x in ln_in; without has_prev ln_in is still read, and ignored: pass any chunk-pair buffer);
// also xg = bf16(x_new * g_next) and the chunk pairs of x_new -> ln_out (a buffer other than ln_in).
// m_real (all three; device, nullable): number of leading rows that hold data; row tiles at or
// beyond it are skipped and rows beyond it are neither computed on nor stored (M stays the
// upper bound the grid is sized for).
hipError_t gemm_ln_sum(hipStream_t st, const bf16* A, int lda, const bf16* W, int M, int d, int K,
                       const float* vecs, const float* ln_in, bool has_prev, float* x, bf16* xg, float* ln_out,
                       const int* m_real = nullptr);
// out bf16 [M,ldo] = act(LN(y) W^T + b) from A = bf16(y * g) [M,d] and the chunk pairs of y
hipError_t gemm_ln_bf16(hipStream_t st, const bf16* A, const bf16* W, int M, int N, int d, const LnFold& f,
                        const float* ln_in, bf16* out, int ldo, bool relu, const int* m_real = nullptr);
// gemm_qkv_append on LN(y)
hipError_t gemm_ln_qkv_append(hipStream_t st, const bf16* A, const bf16* W, int M, int d, const LnFold& f,
                              const float* ln_in, bf16* q_out, bf16* kc, bf16* vc, const int* row_b,
                              const int* row_pos, int H, int Lcap, const int* m_real = nullptr);

// Vocabulary projection fused with per-row statistics.  zd_row [M] receives the logit of the
// draft each row scores (-inf if none).  For every row and every vocabulary tile of
// vocab_tile_cols(M) columns one partial record of kPartF floats is written to
// part[M][n_tiles][kPartF], n_tiles = ceil(V / vocab_tile_cols(M)): {tile max, tile
// arg-max (int bits), sum exp(z - tile max), number of tile logits > zd_row (int bits)}.
// logits (optional, fp32 [M, V]) receives the full rows.  row_draft may be null: no row scores a
// draft (the pre-pass is skipped, zd_row is left untouched and may be null); if logits is null as
// well only max / arg-max are formed (records carry sum 0 and count 0: merged LSE is -inf).
// The product runs on 256 x 256 tiles where those give every CU two or more, or when force_wide is
// set, else on 128 x 128 tiles; the records are per 128 columns either way.
constexpr int kPartF = 4;
constexpr int kRowStats = 8;   // floats per row of merged statistics
int vocab_tile_cols(int M);
hipError_t vocab_stats(hipStream_t st, const bf16* A, const bf16* E, int M, int V, int K,
                       const int* row_draft, float* zd_row, float* part, float* logits, bool force_wide = false);

// ---- per-kernel timing ----------------------------------------------------------------
// While a KernelTimer is set for the calling thread, the next launch of a pass's main kernel (the GEMM,
// attention and vocabulary kernels: SD_LAUNCH_TIMED) records the kernel's own begin and end in its two
// events (the extended launch call), not the moments the stream reaches markers before and after it, and
// says so in `used`.  Launch sites without it leave the timer alone; the caller then brackets the call.
struct KernelTimer {
  hipEvent_t start = nullptr, stop = nullptr;
  bool used = false;
};
void set_kernel_timer(KernelTimer* t);   // nullptr: none
KernelTimer* kernel_timer();
#define SD_LAUNCH_TIMED(kernel, grid, block, smem, st, ...)                                               \
  do {                                                                                                    \
    sd::KernelTimer* kt_ = sd::kernel_timer();                                                            \
    if (kt_ && !kt_->used) {                                                                              \
      kt_->used = true;                                                                                   \
      hipExtLaunchKernelGGL(kernel, grid, block, smem, st, kt_->start, kt_->stop, 0, __VA_ARGS__);        \
    } else {                                                                                              \
      hipLaunchKernelGGL(kernel, grid, block, smem, st, __VA_ARGS__);                                     \
    }                                                                                                     \
  } while (0)

// ---- attn.hip ------------------------------------------------------------------------
struct AttnArgs {
  const bf16* q;  long q_b;                   // q + b*q_b + i*q_row + h*64
  const bf16* k;  long k_b, k_h;              // keys   [key][64]:  k + b*k_b + h*k_h + key*k_row
  const bf16* v;  long v_b, v_h;              // values: v + b*v_b + h*v_h + ...
  bf16* o;        long o_b;                   // o + b*o_b + i*o_row + h*64
  int q_row, k_row, v_row, o_row;             // row strides in elements (the kernel arguments stay small)
  int v_blocked;                              //   1: key-blocked, + vt_off(key, e); whole 32-key chunks are
                                              //      read, capacity % 32 == 0      0: rows, + key*v_row + e
  const int* q_count;                         // [B] queries of sequence b (null: T)
  const int* q_off;                           // [B] first query / output / lim_row row of sequence b (null: b*T,
                                              //     addressed through q_b / o_b); rows are q_row / o_row apart
  const int* lim_row;                         // [rows] visible keys per query (null: lim_seq)
  const int* lim_seq;                         // [B]  visible keys of every query of b
  int T;                                      // max queries per sequence (q_b = T rows apart)
  int H, B;
  int cap;                                    // key rows of one (b, h) arena (multiple of 32); any row below it may be read
  int key_split;                              // 1: the 4 waves of a block split one pair's keys
  // FP8 keys / values (key-blocked values only): k and v then point at E4M3 codes, one byte per element at the
  // same element offsets, and every key's 64-wide vector has its own fp32 scale at index (element offset of the
  // key's row) / 64 of k_scale (keys) / v_scale (values): [b][h][cap] with the arena strides above
  const float* k_scale = nullptr;
  const float* v_scale = nullptr;
};
hipError_t attention(hipStream_t st, const AttnArgs& a);

// ---- skinny.hip: fused kernels for passes of at most 32 rows --------------------------
// Where a kernel takes its input hidden state from: embedding rows (mode 0), raw fp32 rows
// (mode 1) or the LayerNorm of fp32 rows (mode 2), all [R][d].
struct SkSrc {
  int mode;
  const float* xs;
  const bf16* g;
  const bf16* b;
  const int* tok;
  const int* pos;
  const bf16* E;
  const float* pe;
  // np > 0: a sub-layer computed in np slices is still to be summed on top of the state above:
  // hidden = LayerNorm_{g2,b2}(state + pbias + part[0] + .. + part[np-1]), part[p] fp32 [R][d] at
  // part + p * part_stride; the sum itself is stored to xs_out (fp32 [R][d]) by block 0
  const float* part = nullptr;
  int np = 0;
  size_t part_stride = 0;
  const bf16* pbias = nullptr;
  const bf16* g2 = nullptr;
  const bf16* b2 = nullptr;
  float* xs_out = nullptr;
};
bool skinny_supported(int d, int F);
// A weight matrix [N][K] row-major: bf16 values (scale == nullptr), or FP8 E4M3 codes (one byte each)
// with one fp32 scale per row, value = scale[n] * decode(code[n][k]).
struct SkWeight {
  const void* p = nullptr;
  const float* scale = nullptr;
  SkWeight() {}
  SkWeight(const bf16* w) : p(w) {}
  SkWeight(const unsigned char* codes, const float* s) : p(codes), scale(s) {}
};
// codes, scale <- per-row E4M3 quantisation of w [N][K]: scale = max|row| / 448 (1 for a zero row),
// code = nearest-even E4M3 of w / scale.  K % 8 == 0.
hipError_t quantize_rows_e4m3(hipStream_t st, const bf16* w, int N, int K, unsigned char* codes, float* scale);
// The same per-row conversion for cross-attention arenas, a row being one key's 64-wide vector of one head:
// xk [rows][64] -> k8 [rows][64], ksc [rows]; xv key-blocked [rows/8][64][8] -> v8 (same layout), vsc [rows].
// rows % 8 == 0.
hipError_t quantize_cross_kv(hipStream_t st, const bf16* xk, const bf16* xv, long rows, unsigned char* k8,
                             unsigned char* v8, float* ksc, float* vsc);

// ---- resident.hip: the whole verification pass of at most 32 rows as one resident kernel ----
struct RsLayer {
  const bf16 *wqkv, *bqkv, *wo, *bo, *ln1g, *ln1b;
  const bf16 *cwq, *cbq, *cwo, *cbo, *ln2g, *ln2b;
  const bf16 *w1, *b1, *w2, *b2, *ln3g, *ln3b;
};
struct RsArgs {
  int R, T, B, H, V, Lcap, Scap, n_layers;
  const RsLayer* layers;              // device array [n_layers]
  const int *row_tok, *row_pos, *row_b, *row_lim, *row_draft, *seq_rows, *src_len;
  const bf16* E;                      // tied embedding / output matrix [V][d]
  const float* pe;
  float *xs0, *xs1;                   // residual-sum buffers [32][d]
  bf16 *q, *hid;                      // [32][d], [32][F]
  bf16 *kc, *vc;                      // self K/V arenas, layer stride kv_layer
  const bf16 *xk, *xv;                // cross K/V arenas, layer stride xkv_layer
  size_t kv_layer, xkv_layer;
  float *zd, *part, *logits;          // outputs: draft logits [R], tile records, optional logits
  unsigned* bar;                      // kRsBarWords words: [0],[1] arrival counters (alternating
                                      // launches), [16] error flag, [64*(1+h)] wake-up word of helper h
  int parity;                         // which counter this launch uses (the other one is cleared)
  int seq;                            // launch number, never 0
};
constexpr int kRsWorkers = 32;        // workgroups of the resident kernel that run the decoder phases
constexpr int kRsBarWords = 64 * 226;
hipError_t resident_verify(hipStream_t st, const RsArgs& a, int d, int F);
hipError_t skinny_init(int d);
hipError_t skinny_qkv(hipStream_t st, const SkSrc& src, int R, int d, SkWeight W, const bf16* bias, bf16* q,
                      bf16* kc, bf16* vc, const int* row_b, const int* row_pos, int H, int Lcap);
// xs_out = hidden(resid) + attention(a) W^T + bias   (every block recomputes the attention)
hipError_t skinny_attn_o(hipStream_t st, const SkSrc& resid, int R, int d, const AttnArgs& a, SkWeight W,
                         const bf16* bias, float* xs_out);
hipError_t skinny_proj(hipStream_t st, const SkSrc& src, int R, int d, SkWeight W, int N, const bf16* bias,
                       bf16* out, bool relu);
hipError_t skinny_ffn2(hipStream_t st, const SkSrc& resid, int R, int d, const bf16* hid, int F, SkWeight W,
                       const bf16* bias, float* xs_out);
// ---- skinny2.hip: the same passes with sub-layers owned by head / by FFN slice (three kernels per layer) ----
bool sk2_supported(int d, int F);
int sk2_ffn_slices(int F);             // partial results the FFN kernel leaves (at most 16)
constexpr int kSk2MaxParts = 16;       // heads / FFN slices: partial results [R <= 32][d] per kernel
// head h = block h: [hidden from src] -> Q (| K | V, appended) -> attention -> part_out[h] = att_h Wo[:, 64h..64h+63]^T
hipError_t skinny2_head(hipStream_t st, const SkSrc& src, int R, int d, const AttnArgs& a, bool self, const bf16* W,
                        const bf16* bias, bf16* q, bf16* kc, bf16* vc, const int* row_b, const int* row_pos, int Lcap,
                        const bf16* Wo, float* part_out);
// slice s = block s: part_out[s] = ReLU(hidden W1[s]^T + b1[s]) W2[:, s]^T
hipError_t skinny2_ffn(hipStream_t st, const SkSrc& src, int R, int d, const bf16* W1, const bf16* b1, int F,
                       const bf16* W2, float* part_out);
// draft logits + per-row partial records per 64-column vocabulary tile (n_tiles = ceil(V/64))
hipError_t skinny_vocab(hipStream_t st, const SkSrc& src, int R, int d, SkWeight E, int V, const int* row_draft,
                        float* zd_row, float* part, float* logits);

// ---- misc.hip ------------------------------------------------------------------------
hipError_t build_pos_table(hipStream_t st, float* pe, int n_pos, int d);
hipError_t embed_rows(hipStream_t st, const int* tok, const int* pos, const bf16* E,
                      const float* pe, float* x, bf16* xb, int R, int d);
// x <- LayerNorm(x) * g + b in place (fp32), xb <- bf16(x)
hipError_t layer_norm(hipStream_t st, float* x, const bf16* g, const bf16* b, bf16* xb, int R,
                      int d, const int* m_real = nullptr);
// dst [B*k][d] bf16 <- LayerNorm of the mask-slot rows first(b) + new_rows[b] + s of x (x unchanged),
// first(b) = row_start[b], or b*T when row_start is null
hipError_t layer_norm_slots(hipStream_t st, const float* x, const bf16* g, const bf16* b, bf16* dst,
                            const int* new_rows, const int* row_start, int B, int T, int k, int d);
hipError_t fill_i32(hipStream_t st, int* p, int v, long n);

struct SeqState {       // device arrays of the bound state buffer, all [max_batch] unless noted
  int* tokens;          // [max_batch][tok_pitch] stream u_0..u_j
  int* len;             // j
  int* start;           // j when decoding started (tokens after it are output)
  int* cap;             // j may not exceed this (start + max_new, <= max_tgt)
  int* finished;
  int* cached[2];       // per role: stream positions whose K/V are cached
  int* src_len;
  int* last_draft;      // [max_batch][k_max]
  int* scratch;         // [8] counters since begin: commits, tokens appended, finished sequences, near-tau rows
  int tok_pitch, k_max;
};
// rows of a verification pass: [u_j, drafts]; also stores the drafts for commit
hipError_t assemble_verify(hipStream_t st, const SeqState& s, const RowMap& rm, const int* draft,
                           int B, int k, int V);
// assemble_verify and embed_rows of the same rows in one launch
hipError_t assemble_embed_verify(hipStream_t st, const SeqState& s, const RowMap& rm, const int* draft, int B, int k,
                                 int V, const bf16* E, const float* pe, float* x, bf16* xb, int d);
// rows of a prefill pass (n_mask = 0) or of a drafter pass (stream rows + n_mask [MASK] slots),
// embedded in the same launch; new_rows[b] = stream rows of sequence b in this pass;
// packed: rows of the sequences follow each other without padding (RowMap::row_start is written)
hipError_t assemble_embed_stream(hipStream_t st, const SeqState& s, const RowMap& rm, int role, int B, int T,
                                 int n_mask, int mask_id, int pad_id, int V, int* new_rows, const bf16* E,
                                 const float* pe, float* x, bf16* xb, int d, bool packed);
hipError_t advance_cached(hipStream_t st, const SeqState& s, int role, const int* new_rows, int B);
hipError_t gather_slots(hipStream_t st, const bf16* xb, bf16* dst, const int* new_rows, const int* row_start, int B,
                        int T, int k, int d);
hipError_t encoder_rows(hipStream_t st, const int* src, int* tok, int* pos, int B, int S, int V);
// Encoder rows without padding: sequence b owns rows row_start[b] .. + src_len[b] - 1 (running sum, batch
// order; row_start [B+1]), n_rows[0] = their number; tok / pos / row_b [B*S]: rows beyond n_rows get token 0,
// position 0, sequence -1.
hipError_t encoder_rows_packed(hipStream_t st, const int* src, const int* src_len, int* tok, int* pos, int* row_b,
                               int* row_start, int* n_rows, int B, int S, int V);
// dst [B][S][d] <- packed rows (zeros beyond a sequence's length)
hipError_t unpack_rows(hipStream_t st, const bf16* src, const int* row_start, const int* src_len, bf16* dst, int B,
                       int S, int d);
// Merges the vocabulary partials of each of the B*(k+1) rows of a verification pass into
// row_stats [R][kRowStats] = {max, arg-max, log-sum-exp, draft logit, number of logits above the
// draft's, 0, 0, 0}, then applies the top-beta / tau rule and the leading-accept scan per
// sequence, in one launch (k + 1 <= 32)
// (fail: optional device flag; when set every sequence reports accept_len -1, next_token pad)
hipError_t merge_accept(hipStream_t st, const float* part, const float* zd_row, int n_tiles, float* row_stats,
                        const SeqState& s, int B, int k, int beta, float tau, int pad_id, int* accept_len,
                        int* next_token, const unsigned* fail = nullptr);
// the same merge for the B*k mask-slot rows of a drafter pass, draft[b][s] = their arg-max (pad
// for finished sequences), and cached[drafter][b] += new_rows[b]
// (seq_rows: rows of each sequence in the pass; a sequence without its k slots gets pad drafts)
hipError_t merge_drafts(hipStream_t st, const float* part, int n_tiles, float* row_stats, const SeqState& s, int B,
                        int k, int pad_id, const int* new_rows, const int* seq_rows, int* draft);
// k: block size of the pass whose drafts are being committed (accept_len is clamped to it)
// head-based drafting: input rows of the heads (see misc.hip), fp32 -> bf16 rows, arg-max per head row
hipError_t head_rows(hipStream_t st, const float* x, const bf16* g, const bf16* beta, const int* accept_len, int B, int T,
                     int k, int d, bf16* rows, float* rep);
hipError_t f32_to_bf16(hipStream_t st, const float* src, bf16* dst, long n);
hipError_t merge_head_drafts(hipStream_t st, const float* part, int n_tiles, float* row_stats, const SeqState& s,
                             const int* accept_len, int B, int k, int pad_id, int* draft);
hipError_t commit_rows(hipStream_t st, const SeqState& s, const int* accept_len,
                       const int* next_token, int B, int k, int eos_id, int* n_active);
hipError_t begin_state(hipStream_t st, const SeqState& s, int B, int max_new, int max_tgt,
                       int bos_id);
hipError_t set_stream(hipStream_t st, const SeqState& s, const int* tokens, const int* len, int B,
                      int L_max, int max_new, int max_tgt);
hipError_t rewind_state(hipStream_t st, const SeqState& s, const int* len, int B);
hipError_t set_src_len(hipStream_t st, const SeqState& s, const int* src_len, int B, int S_max);
hipError_t set_cached(hipStream_t st, const SeqState& s, int role, const int* n, int B, int hi);
hipError_t get_output(hipStream_t st, const SeqState& s, int* tokens, int out_cap, int* out_len,
                      int* finished, int B, int pad_id);
// key cache [B][H][Lcap][64] / key-blocked value cache  <->  flat [B][L][d]
hipError_t cache_from_flat(hipStream_t st, bf16* cache, const bf16* flat, int B, int H, int Lcap,
                           int L, bool blocked);
hipError_t cache_to_flat(hipStream_t st, const bf16* cache, bf16* flat, int B, int H, int Lcap,
                         int L, bool blocked);

}  // namespace sd
