/*
 * libspecdec -- MI355X (gfx950) implementation of the draft-then-verify hot path of
 * Speculative Decoding (SpecDec, arXiv 2203.16487).
 *
 * C ABI.  Every pointer marked (device) is device memory owned by the caller; every
 * pointer marked (host) is ordinary host memory.  The library allocates no device memory:
 * weights, workspaces, inputs and outputs are the caller's (the one fixed array that
 * specdec_verify_static uses is part of the loaded code object, not an allocation).  `stream` is a hipStream_t
 * passed as void* (NULL = the null stream).  Calls validate their arguments on the host,
 * enqueue work on `stream` and return without synchronising (except where stated).
 * Return value: SPECDEC_OK or a negative specdec_status; specdec_last_error() gives text.
 * A context is not thread-safe.  All work of one context must be issued on one device.
 *
 * Notation (paper Sec. 2): x source, y^_{<=j} tokens decoded so far, y~_{j+1..j+k} the k
 * drafted tokens, c the bifurcation position.  The decoder input stream of a sequence is
 * u_0 = BOS, u_t = y^_t.  Keys/values of u_0..u_{j-1} are cached; u_j is "pending": it is
 * the first row of the next verification pass.
 *
 * Model storage.  All tensors bf16, matrices [out_features, in_features] row-major
 * (y = x W^T + b).  Tensor order (n = specdec_num_weights):
 *   embed [V,d]                                   (tied: input embedding and output projection)
 *   per encoder layer: attn.wqkv [3d,d], attn.bqkv [3d], attn.wo [d,d], attn.bo [d],
 *                      ln1.g [d], ln1.b [d], ffn.w1 [F,d], ffn.b1 [F], ffn.w2 [d,F],
 *                      ffn.b2 [d], ln2.g [d], ln2.b [d]
 *   per decoder layer: self.wqkv [3d,d], self.bqkv [3d], self.wo [d,d], self.bo [d],
 *                      ln1.g, ln1.b, cross.wq [d,d], cross.bq [d], cross.wkv [2d,d],
 *                      cross.bkv [2d], cross.wo [d,d], cross.bo [d], ln2.g, ln2.b,
 *                      ffn.w1, ffn.b1, ffn.w2, ffn.b2, ln3.g, ln3.b
 * Architecture (the paper only names a 6+6 Transformer of 512/2048, Sec. 4.1): post-LN
 * sublayers, LayerNorm eps 1e-5, interleaved sinusoidal positions from 0, embeddings scaled
 * by sqrt(d), scores scaled by 1/sqrt(64), ReLU.  d_model = 64 * n_heads.
 */
#ifndef SPECDEC_H
#define SPECDEC_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct specdec_ctx specdec_ctx; /* opaque, host side */

typedef enum {
  SPECDEC_OK = 0,
  SPECDEC_ERR_INVALID_ARG = -1, /* NULL pointer, value out of range */
  SPECDEC_ERR_BAD_STATE = -2,   /* call order: model/state not bound, begin not called ... */
  SPECDEC_ERR_TOO_LARGE = -3,   /* exceeds the limits given at create / buffer too small */
  SPECDEC_ERR_HIP = -4,         /* a HIP call failed */
  SPECDEC_ERR_NO_DEVICE = -5    /* no usable GPU */
} specdec_status;

typedef enum { SPECDEC_VERIFIER = 0, SPECDEC_DRAFTER = 1 } specdec_role;

typedef struct {
  int32_t enc_layers, dec_layers, d_model, n_heads, d_ffn, vocab;
  int32_t bos_id, eos_id, pad_id, mask_id;
} specdec_model_desc;

typedef struct {
  int32_t max_batch; /* sequences decoded together                                  */
  int32_t k_max;     /* largest block size k (paper uses 10..30, Table 3); <= 31     */
  int32_t max_src;   /* longest source (encoder memory rows per sequence)            */
  int32_t max_tgt;   /* longest decoder stream: j <= max_tgt                         */
} specdec_limits;

enum { SPECDEC_ROW_STATS = 8 }; /* floats per row reported by specdec_get_row_stats */
enum { SPECDEC_COUNTERS = 8 };  /* int32 words reported by specdec_get_counters */

/* Kernel-path switches of a context (specdec_configure), value 0 or 1. */
typedef enum {
  SPECDEC_OPT_SMALL_BATCH_KERNELS = 0, /* default 1: passes of at most 32 rows use the fused small-batch kernels */
  SPECDEC_OPT_LN_FOLD = 1,             /* default 1: decoder LayerNorms folded into the projections around them  */
  SPECDEC_OPT_RESIDENT = 2,            /* default 0: passes of at most 32 rows run as ONE resident kernel        */
  SPECDEC_OPT_SLICED_SUBLAYERS = 3,    /* default 0: the small-batch kernels own sub-layers by output column (six
                                          kernels per layer); 1: by head / FFN slice (three per layer; measured
                                          slower: 8-16 workgroups cannot pull a layer's weights fast enough)      */
  SPECDEC_OPT_FP8_WEIGHTS = 4,         /* default 0.  1, set BEFORE specdec_workspace_bytes and specdec_bind_model:
                                          the model keeps a second copy of its decoder projection matrices (self
                                          QKV, self O, cross Q, cross O, FFN W1, W2) and of the tied output matrix
                                          as FP8 E4M3 codes (OCP 8-bit format: 1-4-3, bias 7, largest value 448, no
                                          infinities) with one fp32 scale per output row, s_n = max_k |w_nk| / 448,
                                          code = nearest-even E4M3 of w_nk / s_n, written by a kernel at bind time.
                                          Passes of at most 32 rows (where weight bytes bound the verification pass
                                          of Sec. 2) then stream the codes -- half the bytes -- turn them into bf16
                                          operands in registers and apply s_n to the fp32 sum:
                                          y_n = s_n * sum_k q_nk h_k + b_n.  This changes the model: its results are
                                          those of the model whose matrices are s_n * q_nk, not of the bf16 one.
                                          Larger passes, the drafter's pass, the encoder, the cross K/V projection
                                          and the input embedding rows keep the bf16 matrices; the RESIDENT and
                                          SLICED_SUBLAYERS paths refuse such a model.                               */
  SPECDEC_OPT_FP8_CROSS_KV = 5,        /* default 0.  1, set BEFORE specdec_workspace_bytes and specdec_bind_model:
                                          the cross-attention keys and values of the model (computed once per input
                                          by specdec_encode / specdec_set_memory, read by every pass of Sec. 2: most
                                          of the bytes of a pass when the source is long) are also stored as E4M3
                                          codes, every key's and every value's 64-wide per-head vector with its own
                                          fp32 scale (max |x| / 448), converted from the bf16 arenas right after they
                                          are written.  Every decoder pass of that model (verification, prefill,
                                          drafting) then reads the codes: score = k_scale * (codes . q),
                                          out += (p * v_scale) * codes.  Changes the model like FP8_WEIGHTS does;
                                          the two options are independent.  Refused by RESIDENT / SLICED_SUBLAYERS. */
  SPECDEC_OPT_WIDE_VOCAB_TILES = 6     /* default 0: the vocabulary projection of a pass of more than 32 rows takes
                                          its 256 x 256 tiles only where they give every compute unit two or more
                                          (the batched passes), else 128 x 128 tiles.  1: 256 x 256 tiles in every
                                          such pass (so that the wide kernel can be checked on small shapes).     */
} specdec_option;

/* ---- life cycle -------------------------------------------------------------------- */
int specdec_create(specdec_ctx** out, const specdec_limits* limits); /* host only */
void specdec_destroy(specdec_ctx* ctx);
const char* specdec_last_error(const specdec_ctx* ctx); /* (host) valid until the next call */
/* Chooses between kernel paths that compute the same pass (all are parity-tested against each other);
 * takes effect from the next specdec_verify / specdec_draft / specdec_prefill.  SPECDEC_OPT_FP8_WEIGHTS and
 * SPECDEC_OPT_FP8_CROSS_KV are the exception on both counts: they select a storage format, and are read by
 * specdec_workspace_bytes and specdec_bind_model.  Host only. */
int specdec_configure(specdec_ctx* ctx, int32_t option, int32_t value);

/* Number of weight tensors of a model and the shape of tensor idx (cols = 1 for vectors). */
int specdec_num_weights(const specdec_model_desc* desc, int32_t* out);
int specdec_weight_shape(const specdec_model_desc* desc, int32_t idx, int64_t* rows, int64_t* cols);

/* Sequence state (token streams, lengths, flags, per-step scratch shared by both models):
 * size query, then bind a (device) buffer of at least that size, 256-byte aligned. */
int specdec_state_bytes(const specdec_ctx* ctx, size_t* out);
int specdec_bind_state(specdec_ctx* ctx, void* state /*device*/, size_t bytes);

/* Per-model workspace (KV arenas, cross-attention K/V, activations, position table). */
int specdec_workspace_bytes(const specdec_ctx* ctx, const specdec_model_desc* desc, size_t* out);
/* weights: (host) array of n_weights (device) pointers in the order above.  The workspace
 * is (device), 256-byte aligned.  Builds the position table on `stream`; also copies a small
 * table of layer pointers into the workspace with a synchronous host-to-device copy.
 * The weight tensors are used in place and must hold their final values when this is called:
 * kernels on `stream` read them here to derive, into the workspace, the per-column vectors with
 * which each decoder LayerNorm is folded into the projections around it (sums of gain x weight
 * and shift x weight over the input dimension).  Bind again after changing weights. */
int specdec_bind_model(specdec_ctx* ctx, specdec_role role, const specdec_model_desc* desc,
                       const void* const* weights, int32_t n_weights, void* workspace,
                       size_t workspace_bytes, void* stream);

/* ---- per batch ---------------------------------------------------------------------- */
/* Start decoding B sequences: every stream = [BOS], j = 0, nothing cached, not finished.
 * max_new = cap on tokens committed per sequence (the paper's "termination condition",
 * Sec. 2, is EOS; a length cap is the usual second one). */
int specdec_begin(specdec_ctx* ctx, int32_t B, int32_t max_new, void* stream);

/* Encoder pass of every bound model over src (device int32 [B, S_max], right-padded;
 * src_len device int32 [B], 1 <= src_len <= S_max <= max_src), then the cross-attention
 * keys/values of every decoder layer.  Runs once per input, not per iteration (Sec. 3.1.2). */
int specdec_encode(specdec_ctx* ctx, const int32_t* src, const int32_t* src_len, int32_t S_max,
                   void* stream);

/* Instead of specdec_encode: take a given encoder memory (device bf16 [B, S_max, d]) for one
 * model and compute that model's cross-attention keys/values from it. */
int specdec_set_memory(specdec_ctx* ctx, specdec_role role, const void* memory,
                       const int32_t* src_len, int32_t S_max, void* stream);

/* Replace the streams by given ones: tokens device int32 [B, L_max+1] holds u_0..u_j per
 * sequence, len device int32 [B] holds j (0 <= j <= L_max <= max_tgt).  After this call no
 * model has anything cached for these streams (cached lengths 0) unless a cache is loaded
 * with specdec_load_cache.  The max_new cap counts tokens committed after this call. */
int specdec_set_stream(specdec_ctx* ctx, const int32_t* tokens, const int32_t* len, int32_t L_max,
                       void* stream);
/* Load self-attention keys/values of u_0..u_{n-1} for one model: k_cache, v_cache device
 * bf16 [dec_layers, B, L_max, d]; n device int32 [B] (n <= j for the verifier, n <= j+1 for
 * the drafter).  Rows at and beyond n are ignored.  The caller vouches that the loaded rows
 * cover the stream (n = j for the verifier, n >= j for the drafter); the device checks it:
 * until specdec_prefill has cached the rest, specdec_verify reports accept_len -1 / next_token
 * pad_id for a sequence with n < j, and specdec_draft returns pad_id drafts for a sequence with
 * more than one uncached stream token. */
int specdec_load_cache(specdec_ctx* ctx, specdec_role role, const void* k_cache,
                       const void* v_cache, const int32_t* n, int32_t L_max, void* stream);

/* One call for "decoding resumes from this prefix": specdec_set_stream(tokens, len, L_max) followed
 * by specdec_load_cache(role, k_cache, v_cache, n = len, L_max).  The streams are shared by both
 * models, so the other model has nothing cached afterwards (load its cache, or prefill it). */
int specdec_set_prefix(specdec_ctx* ctx, specdec_role role, const int32_t* tokens, const int32_t* len,
                       int32_t L_max, const void* k_cache, const void* v_cache, void* stream);

/* Cache the keys/values of every stream token a model has not cached yet (u_0..u_{j-1} for
 * the verifier, u_0..u_j for the drafter) with causal decoder passes of up to k_max+1 rows
 * per sequence.  Needed after specdec_set_stream unless a cache is loaded. */
int specdec_prefill(specdec_ctx* ctx, specdec_role role, void* stream);

/* ---- the hot path -------------------------------------------------------------------- */
/* Spec-Drafter inference (Sec. 3.1.3, Eq. 7): append k [MASK] slots to the stream, one
 * non-autoregressive decoder pass, argmax per slot -> draft device int32 [B, k].  Stream
 * tokens the drafter has not cached yet are processed (causally) in the same pass and
 * cached; mask slots attend to the whole stream and to all k slots.
 * logits_or_null: optional device fp32 [B, k, V] receiving the slots' logits (parity mode; slow). */
int specdec_draft(specdec_ctx* ctx, int32_t k, int32_t* draft, float* logits_or_null, void* stream);

/* Head-based drafting, the cheap drafter the paper compares the Spec-Drafter with (Sec. 2 "Draft",
 * Table 2 first row: k - 1 feed-forward heads on top of the target model, sharing its attention).
 * specdec_bind_draft_heads: n_heads residual feed-forward blocks of the verifier's widths, stacked
 * (device bf16): w1 [n_heads * F, d], b1 [n_heads * F], w2 [n_heads, d, F], b2 [n_heads * d];
 * used in place.  specdec_draft_heads, called after specdec_verify (before or after
 * specdec_commit of the same pass): with h_b the verifier's final hidden state on the bifurcation
 * row accept_len[b] of that pass (the row whose arg-max is next_token),
 *   draft[b][i] = arg-max of  E (h_b + W2_i relu(W1_i h_b + b1_i) + b2_i),   i = 0 .. k-1,
 * the drafts of the positions after next_token: the input of the next specdec_verify once this
 * pass is committed.  pad_id for finished sequences.  k <= n_heads.  The projection is the
 * verifier's tied output matrix.  Overwrites the row statistics of the verification pass.
 * logits_or_null: optional device fp32 [B, k, V] (parity mode). */
int specdec_bind_draft_heads(specdec_ctx* ctx, int32_t n_heads, const void* w1, const void* b1, const void* w2,
                             const void* b2);
int specdec_draft_heads(specdec_ctx* ctx, const int32_t* accept_len, int32_t k, int32_t* draft,
                        float* logits_or_null, void* stream);

/* Verification (Sec. 2 Eq. 1-3; Sec. 3.2 Eq. 8-10): one KV-cached pass of the verifier's
 * decoder over rows [u_j, y~_{j+1}, .., y~_{j+k}] (causal; keys/values of the rows are
 * appended after the cached ones), vocabulary projection and log-softmax statistics fused
 * with the acceptance test.  Draft i is accepted iff drafts 1..i-1 were and, on row i-1,
 *   log P(y~) >= log P(beta-th ranked token)   and   log P(top-1) - log P(y~) <= tau.
 * beta = 1, tau = 0 is the strict top-1 rule; 0 <= k <= k_max, 1 <= beta <= vocab, tau >= 0.
 * Outputs (device int32 [B]):
 *   accept_len = number of accepted drafts a (= c - 1),
 *   next_token = the verifier's arg-max token on row a (lowest index among maxima); when all
 *   k drafts are accepted this is the token after the last draft.
 * Finished sequences report accept_len 0 and next_token pad_id.
 * k = 0 (draft may be null) is one plain autoregressive step: accept_len = 0 and next_token is
 * the verifier's greedy token (the baseline of Sec. 2 on the same kernels).
 * With SPECDEC_OPT_RESIDENT set (specdec_configure), passes of at most 32
 * rows run as one resident kernel whose workgroups meet at bounded grid barriers; should a
 * barrier time out (never expected), every sequence reports accept_len -1 and next_token
 * pad_id, specdec_commit then changes nothing, and the condition lasts until the next
 * specdec_begin.
 * logits_or_null: optional device fp32 [B, k+1, V] receiving every row's logits (parity
 * mode; slow).  Does not change any length: calling it twice gives the same result. */
int specdec_verify(specdec_ctx* ctx, const int32_t* draft, int32_t k, int32_t beta, float tau,
                   int32_t* accept_len, int32_t* next_token, float* logits_or_null, void* stream);

/* specdec_verify for callers that cannot allocate device memory or hand over a workspace for the
 * pass's scratch (code under HIP graph capture, tight serving loops, harnesses that forbid
 * hipMalloc): the vocabulary partial records, draft logits and row statistics of the pass live in
 * a static device array inside the library (5.6 MiB per GPU, held until the process ends)
 * instead of the bound workspace.  Same arguments, same results, no allocation of any kind.
 * Limits: B * (k + 1) <= 1408 rows and rows x vocabulary tiles (128 columns; 64 for passes of at
 * most 32 rows) <= 1408 x 256, else SPECDEC_ERR_TOO_LARGE.  Every call on a GPU shares that GPU's
 * array: calls that overlap on one GPU (two streams, two contexts) race; specdec_get_row_stats
 * after it reads the array, so it must precede the next such call. */
int specdec_verify_static(specdec_ctx* ctx, const int32_t* draft, int32_t k, int32_t beta, float tau,
                          int32_t* accept_len, int32_t* next_token, float* logits_or_null, void* stream);

/* Commit (Eq. 3): append y~_{j+1..j+a} and next_token to each stream, stop a sequence after
 * its first EOS or at its cap; j advances by the number of tokens appended, which also is
 * the number of this pass's cache rows that become valid -- rejected rows are simply left
 * beyond j (rollback moves no data).  Uses the drafts of the latest specdec_verify.
 * n_active_or_null: optional device int32 [1] receiving the number of unfinished sequences. */
int specdec_commit(specdec_ctx* ctx, const int32_t* accept_len, const int32_t* next_token,
                   int32_t* n_active_or_null, void* stream);

/* Roll sequences back: j_b <- min(j_b, len[b]) (len device int32 [B]); cached lengths are cut
 * to match and a sequence whose j drops below its cap is unfinished again.  Like the
 * rollback inside commit this moves no data: rows beyond j are simply dead. */
int specdec_rewind(specdec_ctx* ctx, const int32_t* len, void* stream);

/* ---- read back ----------------------------------------------------------------------- */
/* tokens device int32 [B, out_cap]: tokens committed since begin / set_stream (right-padded
 * with pad_id); out_len device int32 [B]; finished_or_null device int32 [B]. */
int specdec_get_output(specdec_ctx* ctx, int32_t* tokens, int32_t out_cap, int32_t* out_len,
                       int32_t* finished_or_null, void* stream);
/* Cached self-attention keys/values of one model, rows [0, L) of every sequence, in the
 * layout of specdec_load_cache ([dec_layers, B, L, d] bf16).  Rows beyond a sequence's
 * cached length hold whatever the last pass wrote there. */
int specdec_get_cache(specdec_ctx* ctx, specdec_role role, void* k_cache, void* v_cache, int32_t L,
                      void* stream);
/* Encoder memory of one model after specdec_encode: device bf16 [B, S_max, d], zeros in the rows beyond a
 * sequence's source length (the encoder itself runs on the sources' tokens only, without padding rows).
 * SPECDEC_ERR_BAD_STATE if the memory in use came from specdec_set_memory. */
int specdec_get_memory(specdec_ctx* ctx, specdec_role role, void* memory, void* stream);
/* Per-row statistics of the latest specdec_verify, device fp32 [B, k+1, SPECDEC_ROW_STATS]:
 * {max logit, arg-max (as float), log-sum-exp, logit z_d of the draft scored on this row (-inf
 * on the last row), number of logits strictly larger than z_d (as float), 0, 0, 0}.
 * log P(token) = logit - log-sum-exp. */
int specdec_get_row_stats(specdec_ctx* ctx, float* stats, void* stream);
/* The same for the k mask-slot rows of the latest specdec_draft, device fp32 [B, k, SPECDEC_ROW_STATS]:
 * {max logit, arg-max (as float), log-sum-exp (finite only if that pass wrote logits), -inf, 0, 0, 0, 0}. */
int specdec_get_draft_stats(specdec_ctx* ctx, float* stats, void* stream);
/* Counters since specdec_begin, device int32 [SPECDEC_COUNTERS]: {specdec_commit calls, tokens
 * appended by them, sequences finished at the latest commit, verification rows (up to and including
 * the bifurcation row, summed over specdec_verify calls) whose tau test had a margin
 * |tau - (log P(top-1) - log P(draft))| <= 1e-2, 0, 0, 0, 0}.  Mean tokens per iteration (the paper's
 * Tok., Sec. 3.1.1 Eq. 4) = tokens appended / (commits x B). */
int specdec_get_counters(specdec_ctx* ctx, int32_t* counters, void* stream);

/* The bind-time FP8 conversion of SPECDEC_OPT_FP8_WEIGHTS as a call of its own (so that the stored
 * codes can be inspected): w device bf16 [N, K] row-major, K % 8 == 0 -> codes device uint8 [N, K]
 * (8-byte aligned), scale device fp32 [N]; scale[n] = max_k |w[n][k]| / 448 (1 for an all-zero row),
 * codes[n][k] = nearest E4M3 code (ties to the even mantissa, saturating at 448) of w[n][k] / scale[n],
 * every operation in correctly rounded fp32.  Stateless; ctx only receives the error text. */
int specdec_quantize_rows(specdec_ctx* ctx, const void* w, int64_t N, int64_t K, void* codes, float* scale,
                               void* stream);

/* ---- timing of one kernel kind ----------------------------------------------------------- */
/* While a kind is selected every launch of that kernel is timed by a pair of HIP events on the launch
 * stream (up to 4096 launches between two reads; later ones are not recorded): for the GEMM, attention and
 * vocabulary kernels of passes of more than 32 rows the pair holds the kernel's own begin and end, for the
 * other kernels the moments the stream reaches a marker before and after the launch (the hand-over from the
 * launch before is then inside).
 * specdec_profile_read waits for the recorded events (it synchronises on them), returns their
 * summed duration in milliseconds and their number, and clears the record. */
typedef enum {
  SPECDEC_KIND_NONE = -1,
  SPECDEC_KIND_GEMM_F32 = 0,   /* projections with fp32 output + residual (O, cross-O, FFN2) */
  SPECDEC_KIND_GEMM_BF16 = 1,  /* projections with bf16 output (cross-Q, FFN1)               */
  SPECDEC_KIND_GEMM_QKV = 2,   /* self-attention projection with KV append                  */
  SPECDEC_KIND_ATTN = 3,       /* self- and cross-attention                                 */
  SPECDEC_KIND_VOCAB = 4,      /* fused vocabulary projection + row statistics              */
  SPECDEC_KIND_LN = 5,
  SPECDEC_KIND_ACCEPT = 6,
  SPECDEC_KIND_OTHER = 7,
  SPECDEC_KIND_RESIDENT = 8,   /* whole decoder pass + vocabulary tiles of a small batch, one kernel */
  SPECDEC_KIND_COUNT = 9
} specdec_kernel_kind;
int specdec_profile_select(specdec_ctx* ctx, int32_t kind);
int specdec_profile_read(specdec_ctx* ctx, double* total_ms /*host*/, int32_t* launches /*host*/);

#ifdef __cplusplus
}
#endif
#endif /* SPECDEC_H */
