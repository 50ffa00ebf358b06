// C ABI of libspecdec: context, argument checks, workspace layout and the launch sequence
// of every entry point declared in include/specdec.h.
#include <hip/hip_runtime.h>

#include <cmath>
#include <cstdarg>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <new>
#include <vector>

#include "../../include/specdec.h"
#include "kernels.h"

using sd::bf16;

namespace {

struct EncLayer {
  const bf16 *wqkv, *bqkv, *wo, *bo, *ln1g, *ln1b, *w1, *b1, *w2, *b2, *ln2g, *ln2b;
};
struct DecLayer {
  const bf16 *wqkv, *bqkv, *wo, *bo, *ln1g, *ln1b;
  const bf16 *cwq, *cbq, *cwkv, *cbkv, *cwo, *cbo, *ln2g, *ln2b;
  const bf16 *w1, *b1, *w2, *b2, *ln3g, *ln3b;
};

// LayerNorm folded into the projections that read its output: ln3 of the layer below -> wqkv
// (unused in layer 0), ln1 -> cwq, ln2 -> w1.
struct LnFolds {
  sd::LnFold qkv, cq, w1;
  const float *vo, *vco, *v2;   // column vectors of the three residual sums (wo, cwo, w2), [3][d] each
};

// FP8 copies of the matrices the small-batch kernels stream (codes + per-row scales)
struct Fp8Layer {
  sd::SkWeight wqkv, wo, cwq, cwo, w1, w2;
};

struct Model {
  bool bound = false;
  bool has_memory = false;
  bool enc_packed = false;   // exb holds the memory of the latest specdec_encode as packed rows
  specdec_model_desc d{};
  const bf16* embed = nullptr;
  std::vector<EncLayer> enc;
  std::vector<DecLayer> dec;
  // workspace
  float* pe = nullptr;       // [n_pos][d]
  bf16 *kc = nullptr, *vc = nullptr;   // [Ld][Bmax][H][Lcap][64]
  bf16 *xk = nullptr, *xv = nullptr;   // [Ld][Bmax][H][Scap][64]
  float* x = nullptr;        // [Rmax][d] residual stream
  float* x2 = nullptr;       // [32][d] second residual buffer of the fused small-batch path
  float* skp = nullptr;      // [2][kSk2MaxParts][32][d] partial results of the sliced small-batch kernels
  unsigned char* w8 = nullptr;   // E4M3 codes of every decoder layer's six matrices, then the embedding (or null)
  float* w8s = nullptr;          // their row scales, same order
  bool fp8 = false;              // bound with SPECDEC_OPT_FP8_WEIGHTS: passes of at most 32 rows stream w8
  bool kv8 = false;              // bound with SPECDEC_OPT_FP8_CROSS_KV: cross-attention reads xk8 / xv8
  unsigned char *xk8 = nullptr, *xv8 = nullptr;   // E4M3 codes of xk / xv, same layouts
  float *xks = nullptr, *xvs = nullptr;           // one scale per (layer, sequence, head, key)
  std::vector<Fp8Layer> dec8;
  sd::SkWeight embed8;
  float* hx = nullptr;       // [Bmax*k_max][d] head-based drafting: the hidden state each head adds to, then its output
  bool skinny_ready = false;
  sd::RsLayer* rs_layers = nullptr;   // device copy of the decoder layers' pointers (resident kernel)
  unsigned* rs_bar = nullptr;         // barrier counters + error flag of the resident kernel
  int rs_parity = 0;
  int rs_seq = 0;
  bf16* xb = nullptr;        // [Rmax][d]
  float* lnp[2] = {nullptr, nullptr};   // [rows][d/64 rounded up to even][2] chunk pairs of the two latest residual sums
  float* fold = nullptr;     // per decoder layer: cs and bf vectors of wqkv, cwq, w1 (LayerNorm folded)
  std::vector<LnFolds> folds;
  bf16* q = nullptr;         // [Rmax][d]
  bf16* att = nullptr;       // [Rmax][d]
  bf16* hid = nullptr;       // [Rmax][F]
  float* part = nullptr;     // [Rmax][n_tiles][kPartF]
  float* row_stats = nullptr;  // [Rmax][kRowStats]
  float* zd = nullptr;       // [Rmax] logit of the draft each row scores
  bf16* slots = nullptr;     // [Bmax*k_max][d] final hidden states of the drafter's mask slots
  int* new_rows = nullptr;   // [Bmax] stream rows of the current prefill / draft pass
  // encoder activations, rows = Bmax * Scap
  float* ex = nullptr;
  bf16 *exb = nullptr, *eqkv = nullptr, *eatt = nullptr, *ehid = nullptr;
  int *etok = nullptr, *epos = nullptr;
  int *erow_b = nullptr, *erow_start = nullptr, *en_rows = nullptr;   // packed encoder rows: owner, first row per sequence, count
  sd::RowMap rm{};
  size_t kv_layer = 0, xkv_layer = 0;  // elements per layer of the arenas
};

}  // namespace

struct specdec_ctx {
  specdec_limits lim{};
  int Lcap = 0, Scap = 0, Tmax = 0, n_pos = 0;
  bool state_bound = false;
  sd::SeqState st{};
  Model m[2];
  int B = 0;          // batch of the current begin()
  int max_new = 0;
  int last_T = 0;     // rows per sequence (k + 1) of the latest verify (0: none)
  int last_k_draft = 0;   // k of the latest drafter pass (0: none)
  const float* last_row_stats = nullptr;   // merged row statistics of the latest verify
  // final hidden states of the latest verify: rows [B*T][d], normalised, or still to be normalised with (fin_g, fin_b)
  const float* fin_x = nullptr;
  const bf16 *fin_g = nullptr, *fin_b = nullptr;
  // drafting heads on top of the verifier (stacked): w1 [n*F,d], b1 [n*F], w2 [n][d,F], b2 [n*d]
  int n_draft_heads = 0;
  const bf16 *hw1 = nullptr, *hb1 = nullptr, *hw2 = nullptr, *hb2 = nullptr;
  bool last_draft_by_heads = false;
  int S_cur = 0;      // S_max of the current memory
  int uncached_ub[2] = {0, 0};
  bool trusted[2] = {false, false};
  // event timing of one kernel kind
  int prof_kind = SPECDEC_KIND_NONE;
  std::vector<hipEvent_t> prof_ev;
  int prof_used = 0;
  bool no_skinny = false;   // SPECDEC_OPT_SMALL_BATCH_KERNELS = 0: always take the general kernels
  bool no_ln_fold = false;  // SPECDEC_OPT_LN_FOLD = 0: LayerNorm as a pass of its own between the GEMMs
  bool resident = false;    // SPECDEC_OPT_RESIDENT = 1: small batches run the decoder pass as one resident kernel
  bool sliced = false;      // SPECDEC_OPT_SLICED_SUBLAYERS = 1: small-batch sub-layers owned by head / FFN slice
  bool fp8 = false;         // SPECDEC_OPT_FP8_WEIGHTS = 1: models bound from now on keep E4M3 copies for small batches
  bool fp8_kv = false;      // SPECDEC_OPT_FP8_CROSS_KV = 1: models bound from now on keep E4M3 cross keys / values
  bool wide_vocab = false;  // SPECDEC_OPT_WIDE_VOCAB_TILES = 1: 256 x 256 vocabulary tiles in every pass of more than 32 rows
  char err[512] = {0};
};

namespace {

int fail(const specdec_ctx* c, int code, const char* fmt, ...) {
  if (c) {
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(const_cast<specdec_ctx*>(c)->err, sizeof(c->err), fmt, ap);
    va_end(ap);
  }
  return code;
}
#define HIPCHK(c, expr)                                                                   \
  do {                                                                                    \
    hipError_t e_ = (expr);                                                               \
    if (e_ != hipSuccess)                                                                 \
      return fail(c, SPECDEC_ERR_HIP, "%s failed: %s", #expr, hipGetErrorString(e_));     \
  } while (0)

constexpr int kProfPairs = 4096;
// One launch of the selected kind between two events.  Where the launcher times its main kernel itself
// (sd::KernelTimer) the pair holds that kernel's own begin and end; else the pair brackets the call on the
// stream (and then also holds the hand-over from the launch before).
inline bool prof_begin(specdec_ctx* c, int kind, hipStream_t st, sd::KernelTimer& t) {
  if (c->prof_kind != kind || c->prof_used + 2 > (int)c->prof_ev.size()) return false;
  if (hipEventRecord(c->prof_ev[c->prof_used], st) != hipSuccess) return false;
  t.start = c->prof_ev[c->prof_used];
  t.stop = c->prof_ev[c->prof_used + 1];
  t.used = false;
  sd::set_kernel_timer(&t);
  return true;
}
inline void prof_end(specdec_ctx* c, hipStream_t st, const sd::KernelTimer& t) {
  sd::set_kernel_timer(nullptr);
  if (!t.used) (void)hipEventRecord(c->prof_ev[c->prof_used + 1], st);
  c->prof_used += 2;
}
// launch `expr` (a kernels.h launcher on stream st) as kernel kind `kind`
#define LAUNCH(c, kind, st, expr)            \
  do {                                       \
    sd::KernelTimer kt_;                     \
    bool p_ = prof_begin(c, kind, st, kt_);  \
    hipError_t le_ = (expr);                 \
    if (p_) prof_end(c, st, kt_);            \
    if (le_ != hipSuccess)                   \
      return fail(c, SPECDEC_ERR_HIP, "%s failed: %s", #expr, hipGetErrorString(le_)); \
  } while (0)

bool desc_ok(const specdec_model_desc* d) {
  return d && d->enc_layers >= 0 && d->dec_layers >= 1 && d->n_heads >= 1 && d->n_heads <= 32 &&
         d->d_model == 64 * d->n_heads && d->d_ffn >= 64 && d->d_ffn % 64 == 0 && d->d_ffn <= 16384 &&
         d->vocab >= 8 && d->vocab <= (1 << 24) && d->bos_id >= 0 && d->bos_id < d->vocab &&
         d->eos_id >= 0 && d->eos_id < d->vocab && d->pad_id >= 0 && d->pad_id < d->vocab &&
         d->mask_id >= 0 && d->mask_id < d->vocab;
}
constexpr int kEncT = 12, kDecT = 20;
int n_weights(const specdec_model_desc* d) { return 1 + kEncT * d->enc_layers + kDecT * d->dec_layers; }

void weight_shape(const specdec_model_desc* d, int idx, int64_t* r, int64_t* c) {
  const int64_t D = d->d_model, F = d->d_ffn;
  if (idx == 0) { *r = d->vocab; *c = D; return; }
  idx -= 1;
  static const int enc_kind[kEncT] = {0, 1, 2, 3, 3, 3, 4, 5, 6, 3, 3, 3};
  // kinds: 0 [3d,d] 1 [3d] 2 [d,d] 3 [d] 4 [F,d] 5 [F] 6 [d,F] 7 [2d,d] 8 [2d]
  static const int dec_kind[kDecT] = {0, 1, 2, 3, 3, 3, 2, 3, 7, 8, 2, 3, 3, 3, 4, 5, 6, 3, 3, 3};
  int kind;
  if (idx < kEncT * d->enc_layers) kind = enc_kind[idx % kEncT];
  else kind = dec_kind[(idx - kEncT * d->enc_layers) % kDecT];
  switch (kind) {
    case 0: *r = 3 * D; *c = D; break;
    case 1: *r = 3 * D; *c = 1; break;
    case 2: *r = D; *c = D; break;
    case 3: *r = D; *c = 1; break;
    case 4: *r = F; *c = D; break;
    case 5: *r = F; *c = 1; break;
    case 6: *r = D; *c = F; break;
    case 7: *r = 2 * D; *c = D; break;
    default: *r = 2 * D; *c = 1; break;
  }
}

// bump allocator over a (possibly null) base: the same walk sizes and carves a buffer
struct Carver {
  char* base;
  size_t off = 0;
  explicit Carver(void* b) : base(static_cast<char*>(b)) {}
  template <class T>
  T* take(size_t n) {
    off = (off + 255) & ~size_t(255);
    T* p = base ? reinterpret_cast<T*>(base + off) : nullptr;
    off += n * sizeof(T);
    return p;
  }
};

size_t carve_state(const specdec_ctx* c, void* base, sd::SeqState* out) {
  Carver cv(base);
  const size_t Bm = c->lim.max_batch;
  sd::SeqState s{};
  s.tok_pitch = c->lim.max_tgt + 1;
  s.k_max = c->lim.k_max;
  s.tokens = cv.take<int>(Bm * s.tok_pitch);
  s.len = cv.take<int>(Bm);
  s.start = cv.take<int>(Bm);
  s.cap = cv.take<int>(Bm);
  s.finished = cv.take<int>(Bm);
  s.cached[0] = cv.take<int>(Bm);
  s.cached[1] = cv.take<int>(Bm);
  s.src_len = cv.take<int>(Bm);
  s.last_draft = cv.take<int>(Bm * s.k_max);
  s.scratch = cv.take<int>(8);
  if (out) *out = s;
  return (cv.off + 255) & ~size_t(255);
}

size_t carve_model(const specdec_ctx* c, const specdec_model_desc* d, void* base, Model* m) {
  Carver cv(base);
  const size_t Bm = c->lim.max_batch, D = d->d_model, F = d->d_ffn, H = d->n_heads;
  const size_t Rmax = Bm * c->Tmax;
  const size_t n_tiles = (d->vocab + 63) / 64;   // the small-batch path uses 64-column tiles
  Model t;
  t.kv_layer = Bm * H * c->Lcap * 64;
  t.xkv_layer = Bm * H * (size_t)c->Scap * 64;
  t.pe = cv.take<float>((size_t)c->n_pos * D);
  t.kc = cv.take<bf16>(t.kv_layer * d->dec_layers);
  t.vc = cv.take<bf16>(t.kv_layer * d->dec_layers);
  t.xk = cv.take<bf16>(t.xkv_layer * d->dec_layers);
  t.xv = cv.take<bf16>(t.xkv_layer * d->dec_layers);
  t.x = cv.take<float>(Rmax * D);
  t.x2 = cv.take<float>(32 * D);
  t.skp = cv.take<float>((size_t)2 * sd::kSk2MaxParts * 32 * D);
  t.hx = cv.take<float>(Bm * (size_t)c->lim.k_max * D);
  if (c->fp8_kv) {
    t.xk8 = cv.take<unsigned char>(t.xkv_layer * d->dec_layers);
    t.xv8 = cv.take<unsigned char>(t.xkv_layer * d->dec_layers);
    t.xks = cv.take<float>(t.xkv_layer / 64 * d->dec_layers);
    t.xvs = cv.take<float>(t.xkv_layer / 64 * d->dec_layers);
  }
  if (c->fp8) {
    t.w8 = cv.take<unsigned char>((size_t)d->dec_layers * (6 * D * D + 2 * D * F) + (size_t)d->vocab * D);
    t.w8s = cv.take<float>((size_t)d->dec_layers * (7 * D + F) + (size_t)d->vocab);
  }
  t.xb = cv.take<bf16>(Rmax * D);
  t.lnp[0] = cv.take<float>(Rmax * (D / 64 + 1) * 2);
  t.lnp[1] = cv.take<float>(Rmax * (D / 64 + 1) * 2);
  t.fold = cv.take<float>((size_t)d->dec_layers * (2 * (3 * D + D + F) + 9 * D));
  t.q = cv.take<bf16>((Rmax > 32 ? Rmax : 32) * D);
  t.att = cv.take<bf16>(Rmax * D);
  t.hid = cv.take<bf16>((Rmax > 32 ? Rmax : 32) * F);
  t.part = cv.take<float>(Rmax * n_tiles * sd::kPartF);
  t.row_stats = cv.take<float>(Rmax * sd::kRowStats);
  t.zd = cv.take<float>(Rmax);
  t.rm.row_b = cv.take<int>(Rmax);
  t.rm.row_pos = cv.take<int>(Rmax);
  t.rm.row_tok = cv.take<int>(Rmax);
  t.rm.row_lim = cv.take<int>(Rmax);
  t.rm.row_draft = cv.take<int>(Rmax);
  t.rm.seq_rows = cv.take<int>(Bm);
  t.rm.row_start = cv.take<int>(Bm + 1);
  t.slots = cv.take<bf16>(Bm * (size_t)c->lim.k_max * D);
  t.new_rows = cv.take<int>(Bm);
  t.rs_layers = cv.take<sd::RsLayer>(d->dec_layers);
  t.rs_bar = cv.take<unsigned>(sd::kRsBarWords);
  if (d->enc_layers > 0) {
    const size_t Re = Bm * (size_t)c->Scap;
    t.ex = cv.take<float>(Re * D);
    t.exb = cv.take<bf16>(Re * D);
    t.eqkv = cv.take<bf16>(Re * 3 * D);
    t.eatt = cv.take<bf16>(Re * D);
    t.ehid = cv.take<bf16>(Re * F);
    t.etok = cv.take<int>(Re);
    t.epos = cv.take<int>(Re);
    t.erow_b = cv.take<int>(Re);
    t.erow_start = cv.take<int>(Bm + 1);
    t.en_rows = cv.take<int>(1);
  }
  if (m) {
    m->kv_layer = t.kv_layer; m->xkv_layer = t.xkv_layer;
    m->pe = t.pe; m->kc = t.kc; m->vc = t.vc; m->xk = t.xk; m->xv = t.xv;
    m->lnp[0] = t.lnp[0]; m->lnp[1] = t.lnp[1]; m->fold = t.fold;
    m->x = t.x; m->x2 = t.x2; m->skp = t.skp; m->hx = t.hx; m->w8 = t.w8; m->w8s = t.w8s; m->xk8 = t.xk8; m->xv8 = t.xv8; m->xks = t.xks; m->xvs = t.xvs; m->xb = t.xb; m->q = t.q; m->att = t.att; m->hid = t.hid;
    m->part = t.part; m->row_stats = t.row_stats; m->zd = t.zd; m->rm = t.rm;
    m->slots = t.slots; m->new_rows = t.new_rows; m->rs_layers = t.rs_layers; m->rs_bar = t.rs_bar;
    m->ex = t.ex; m->exb = t.exb; m->eqkv = t.eqkv; m->eatt = t.eatt; m->ehid = t.ehid;
    m->etok = t.etok; m->epos = t.epos; m->erow_b = t.erow_b; m->erow_start = t.erow_start; m->en_rows = t.en_rows;
  }
  return (cv.off + 255) & ~size_t(255);
}

inline hipStream_t S(void* s) { return static_cast<hipStream_t>(s); }

// Point a cross-attention launch of layer l at the E4M3 copies of the keys / values (same strides).
inline void cross_fp8(const Model& m, int l, sd::AttnArgs& a) {
  a.k = reinterpret_cast<const bf16*>(m.xk8 + m.xkv_layer * l);
  a.v = reinterpret_cast<const bf16*>(m.xv8 + m.xkv_layer * l);
  a.k_scale = m.xks + m.xkv_layer / 64 * l;
  a.v_scale = m.xvs + m.xkv_layer / 64 * l;
}

// Embedding (unless the caller's row assembly has already written it to m.x / m.xb) + every
// decoder layer over the R = B*T rows described by m.rm.  Leaves the final hidden states in
// m.x (fp32) and m.xb (bf16); with slot_k > 0 (drafter pass) only those of the slot_k mask-slot
// rows per sequence are needed, and they go to m.slots [B*slot_k][d] (bf16) instead.
// packed: the rows of the pass were assembled without padding (m.rm.row_start); R = B*T is then
// only the bound the grids are sized for, and tiles beyond the rows in use return at once.
int decoder_layers(specdec_ctx* c, Model& m, int B, int T, hipStream_t st, bool embedded = false, int slot_k = 0,
                   bool packed = false) {
  const int R = B * T, D = m.d.d_model, F = m.d.d_ffn, H = m.d.n_heads;
  const int Lcap = c->Lcap, Scap = c->Scap;
  const int* m_real = packed ? m.rm.row_start + B : nullptr;
  const int* row_start = packed ? m.rm.row_start : nullptr;
  if (!embedded)
    LAUNCH(c, SPECDEC_KIND_OTHER, st, sd::embed_rows(st, m.rm.row_tok, m.rm.row_pos, m.embed, m.pe, m.x, m.xb, R, D));
  // LayerNorm folded into the GEMMs on both sides of it: m.x holds the un-normalised sum, m.xb
  // that sum times the gain, `pend` the LayerNorm still to be applied to them.
  const bool fold = !c->no_ln_fold;
  const float* pend = nullptr;   // chunk pairs of the sum in m.x (null: m.x is the residual itself)
  int flip = 0;
  auto sum = [&](const bf16* A, int K, const bf16* W, const float* vecs) {
    float* out = m.lnp[flip];
    hipError_t e = sd::gemm_ln_sum(st, A, K, W, R, D, K, vecs, pend ? pend : m.lnp[flip ^ 1], pend != nullptr, m.x, m.xb, out,
                                   m_real);
    pend = out;
    flip ^= 1;
    return e;
  };
  for (int l = 0; l < m.d.dec_layers; ++l) {
    const DecLayer& L = m.dec[l];
    bf16* kc = m.kc + m.kv_layer * l;
    bf16* vc = m.vc + m.kv_layer * l;
    if (fold && l > 0) {
      LAUNCH(c, SPECDEC_KIND_GEMM_QKV, st, sd::gemm_ln_qkv_append(st, m.xb, L.wqkv, R, D, m.folds[l].qkv, pend, m.q, kc,
                                       vc, m.rm.row_b, m.rm.row_pos, H, Lcap, m_real));
    } else {
      LAUNCH(c, SPECDEC_KIND_GEMM_QKV, st, sd::gemm_qkv_append(st, m.xb, L.wqkv, R, D, D, L.bqkv, m.q, kc, vc, m.rm.row_b,
                                    m.rm.row_pos, H, Lcap, m_real));
    }
    sd::AttnArgs a{};
    a.q = m.q; a.q_b = (long)T * D; a.q_row = D;
    a.k = kc; a.k_b = (long)H * Lcap * 64; a.k_h = (long)Lcap * 64; a.k_row = 64;
    a.v = vc; a.v_b = (long)H * Lcap * 64; a.v_h = (long)Lcap * 64; a.v_row = 64; a.v_blocked = 0;
    a.o = m.att; a.o_b = (long)T * D; a.o_row = D;
    a.q_count = m.rm.seq_rows; a.q_off = row_start; a.lim_row = m.rm.row_lim; a.lim_seq = nullptr;
    a.T = T; a.H = H; a.B = B;
    a.key_split = Lcap > 256; a.cap = Lcap;
    LAUNCH(c, SPECDEC_KIND_ATTN, st, sd::attention(st, a));
    if (fold) {
      LAUNCH(c, SPECDEC_KIND_GEMM_F32, st, sum(m.att, D, L.wo, m.folds[l].vo));
      LAUNCH(c, SPECDEC_KIND_GEMM_BF16, st, sd::gemm_ln_bf16(st, m.xb, L.cwq, R, D, D, m.folds[l].cq, pend, m.q, D, false, m_real));
    } else {
      LAUNCH(c, SPECDEC_KIND_GEMM_F32, st, sd::gemm_f32(st, m.att, D, L.wo, R, D, D, L.bo, m.x, m.x, D));
      LAUNCH(c, SPECDEC_KIND_LN, st, sd::layer_norm(st, m.x, L.ln1g, L.ln1b, m.xb, R, D));
      LAUNCH(c, SPECDEC_KIND_GEMM_BF16, st, sd::gemm_bf16(st, m.xb, D, L.cwq, R, D, D, L.cbq, m.q, D, false));
    }
    a.k = m.xk + m.xkv_layer * l; a.k_b = (long)H * Scap * 64; a.k_h = (long)Scap * 64;
    a.v = m.xv + m.xkv_layer * l; a.v_b = (long)H * Scap * 64; a.v_h = (long)Scap * 64; a.v_blocked = 1;
    a.lim_row = nullptr; a.lim_seq = c->st.src_len;
    a.key_split = c->S_cur > 256; a.cap = Scap;
    if (m.kv8) cross_fp8(m, l, a);
    LAUNCH(c, SPECDEC_KIND_ATTN, st, sd::attention(st, a));
    if (fold) {
      LAUNCH(c, SPECDEC_KIND_GEMM_F32, st, sum(m.att, D, L.cwo, m.folds[l].vco));
      LAUNCH(c, SPECDEC_KIND_GEMM_BF16, st, sd::gemm_ln_bf16(st, m.xb, L.w1, R, F, D, m.folds[l].w1, pend, m.hid, F, true, m_real));
      LAUNCH(c, SPECDEC_KIND_GEMM_F32, st, sum(m.hid, F, L.w2, m.folds[l].v2));
      if (l + 1 == m.d.dec_layers) {   // the vocabulary projection reads the normalised rows themselves
        if (slot_k > 0)
          LAUNCH(c, SPECDEC_KIND_LN, st, sd::layer_norm_slots(st, m.x, L.ln3g, L.ln3b, m.slots, m.new_rows, row_start, B, T, slot_k, D));
        else
          LAUNCH(c, SPECDEC_KIND_LN, st, sd::layer_norm(st, m.x, L.ln3g, L.ln3b, m.xb, R, D));
      }
    } else {
      LAUNCH(c, SPECDEC_KIND_GEMM_F32, st, sd::gemm_f32(st, m.att, D, L.cwo, R, D, D, L.cbo, m.x, m.x, D));
      LAUNCH(c, SPECDEC_KIND_LN, st, sd::layer_norm(st, m.x, L.ln2g, L.ln2b, m.xb, R, D));
      LAUNCH(c, SPECDEC_KIND_GEMM_BF16, st, sd::gemm_bf16(st, m.xb, D, L.w1, R, F, D, L.b1, m.hid, F, true));
      LAUNCH(c, SPECDEC_KIND_GEMM_F32, st, sd::gemm_f32(st, m.hid, F, L.w2, R, D, F, L.b2, m.x, m.x, D));
      LAUNCH(c, SPECDEC_KIND_LN, st, sd::layer_norm(st, m.x, L.ln3g, L.ln3b, m.xb, R, D));
    }
  }
  if (slot_k > 0 && !fold) HIPCHK(c, sd::gather_slots(st, m.xb, m.slots, m.new_rows, row_start, B, T, slot_k, D));
  return SPECDEC_OK;
}

// Same pass with the fused small-batch kernels (at most 32 rows).  Returns in `out` where the
// final hidden state comes from (LayerNorm of the last residual sum).
bool skinny_ok(const specdec_ctx* c, const Model& m, int R, int T) {
  return !c->no_skinny && R <= 32 && T <= 32 && sd::skinny_supported(m.d.d_model, m.d.d_ffn) &&
         c->Lcap <= 256 && c->S_cur <= 256;
}

int decoder_layers_skinny(specdec_ctx* c, Model& m, int B, int T, hipStream_t st, sd::SkSrc* out) {
  const int R = B * T, D = m.d.d_model, F = m.d.d_ffn, H = m.d.n_heads;
  const int Lcap = c->Lcap, Scap = c->Scap;
  if (!m.skinny_ready) {
    HIPCHK(c, sd::skinny_init(D));
    m.skinny_ready = true;
  }
  sd::SkSrc cur{0, nullptr, nullptr, nullptr, m.rm.row_tok, m.rm.row_pos, m.embed, m.pe};
  float* freeb = m.x;       // residual-sum buffer not read by the kernel being launched
  float* other = m.x2;
  auto produced = [&](const bf16* g, const bf16* b) {   // freeb now holds the new sum
    cur = sd::SkSrc{2, freeb, g, b, nullptr, nullptr, nullptr, nullptr};
    float* t = freeb; freeb = other; other = t;
  };
  for (int l = 0; l < m.d.dec_layers; ++l) {
    const DecLayer& L = m.dec[l];
    Fp8Layer W;   // the matrices streamed: bf16 as bound, or their E4M3 copies
    if (m.fp8) W = m.dec8[l];
    else { W.wqkv = L.wqkv; W.wo = L.wo; W.cwq = L.cwq; W.cwo = L.cwo; W.w1 = L.w1; W.w2 = L.w2; }
    bf16* kc = m.kc + m.kv_layer * l;
    bf16* vc = m.vc + m.kv_layer * l;
    LAUNCH(c, SPECDEC_KIND_GEMM_QKV, st, sd::skinny_qkv(st, cur, R, D, W.wqkv, L.bqkv, m.q, kc, vc, m.rm.row_b, m.rm.row_pos, H, Lcap));
    sd::AttnArgs a{};
    a.q = m.q; a.q_b = (long)T * D; a.q_row = D;
    a.k = kc; a.k_b = (long)H * Lcap * 64; a.k_h = (long)Lcap * 64; a.k_row = 64;
    a.v = vc; a.v_b = (long)H * Lcap * 64; a.v_h = (long)Lcap * 64; a.v_row = 64; a.v_blocked = 0;
    a.o = nullptr; a.o_b = 0; a.o_row = 0;
    a.q_count = m.rm.seq_rows; a.lim_row = m.rm.row_lim; a.lim_seq = nullptr;
    a.T = T; a.H = H; a.B = B; a.key_split = 0; a.cap = Lcap;
    LAUNCH(c, SPECDEC_KIND_GEMM_F32, st, sd::skinny_attn_o(st, cur, R, D, a, W.wo, L.bo, freeb));
    produced(L.ln1g, L.ln1b);
    LAUNCH(c, SPECDEC_KIND_GEMM_BF16, st, sd::skinny_proj(st, cur, R, D, W.cwq, D, L.cbq, m.q, false));
    a.k = m.xk + m.xkv_layer * l; a.k_b = (long)H * Scap * 64; a.k_h = (long)Scap * 64;
    a.v = m.xv + m.xkv_layer * l; a.v_b = (long)H * Scap * 64; a.v_h = (long)Scap * 64; a.v_blocked = 1;
    a.lim_row = nullptr; a.lim_seq = c->st.src_len; a.cap = Scap;
    if (m.kv8) cross_fp8(m, l, a);
    LAUNCH(c, SPECDEC_KIND_GEMM_F32, st, sd::skinny_attn_o(st, cur, R, D, a, W.cwo, L.cbo, freeb));
    produced(L.ln2g, L.ln2b);
    LAUNCH(c, SPECDEC_KIND_GEMM_BF16, st, sd::skinny_proj(st, cur, R, D, W.w1, F, L.b1, m.hid, true));
    LAUNCH(c, SPECDEC_KIND_GEMM_F32, st, sd::skinny_ffn2(st, cur, R, D, m.hid, F, W.w2, L.b2, freeb));
    produced(L.ln3g, L.ln3b);
  }
  *out = cur;
  return SPECDEC_OK;
}


// The same pass with three kernels per layer: sub-layers owned by head (attention) and by slice of
// the FFN width; each kernel leaves partial results that the next one's prologue sums (fixed order),
// adds bias and residual to, and normalises.  The last layer's FFN runs as two column-owned kernels,
// so that the vocabulary tiles start from a stored sum.
int decoder_layers_sliced(specdec_ctx* c, Model& m, int B, int T, hipStream_t st, sd::SkSrc* out) {
  const int R = B * T, D = m.d.d_model, F = m.d.d_ffn, H = m.d.n_heads;
  const int Lcap = c->Lcap, Scap = c->Scap;
  if (!m.skinny_ready) {
    HIPCHK(c, sd::skinny_init(D));
    m.skinny_ready = true;
  }
  float* S[2] = {m.x, m.x2};
  float* P[2] = {m.skp, m.skp + (size_t)sd::kSk2MaxParts * 32 * D};
  const size_t pstride = (size_t)32 * D;
  int si = 0, pi = 0;
  // the state a kernel starts from once its pending sum (if any) has been stored by the kernel before
  auto resolved = [](const sd::SkSrc& s) {
    if (s.np == 0) return s;
    sd::SkSrc r{2, s.xs_out, s.g2, s.b2, nullptr, nullptr, nullptr, nullptr};
    return r;
  };
  auto with_sum = [&](sd::SkSrc base, const float* part, int np, const bf16* pbias, const bf16* g2, const bf16* b2,
                      float* xs_out) {
    base.part = part; base.np = np; base.part_stride = pstride; base.pbias = pbias; base.g2 = g2; base.b2 = b2;
    base.xs_out = xs_out;
    return base;
  };
  sd::SkSrc cur{0, nullptr, nullptr, nullptr, m.rm.row_tok, m.rm.row_pos, m.embed, m.pe};
  for (int l = 0; l < m.d.dec_layers; ++l) {
    const DecLayer& L = m.dec[l];
    bf16* kc = m.kc + m.kv_layer * l;
    bf16* vc = m.vc + m.kv_layer * l;
    sd::AttnArgs a{};
    a.q = m.q; a.q_b = (long)T * D; a.q_row = D;
    a.k = kc; a.k_b = (long)H * Lcap * 64; a.k_h = (long)Lcap * 64; a.k_row = 64;
    a.v = vc; a.v_b = (long)H * Lcap * 64; a.v_h = (long)Lcap * 64; a.v_row = 64; a.v_blocked = 0;
    a.o = nullptr; a.o_b = 0; a.o_row = 0;
    a.q_count = m.rm.seq_rows; a.lim_row = m.rm.row_lim; a.lim_seq = nullptr;
    a.T = T; a.H = H; a.B = B; a.key_split = 0; a.cap = Lcap;
    LAUNCH(c, SPECDEC_KIND_GEMM_QKV, st, sd::skinny2_head(st, cur, R, D, a, true, L.wqkv, L.bqkv, m.q, kc, vc, m.rm.row_b,
                                      m.rm.row_pos, Lcap, L.wo, P[pi]));
    const sd::SkSrc bsrc = with_sum(resolved(cur), P[pi], H, L.bo, L.ln1g, L.ln1b, S[si]);
    a.k = m.xk + m.xkv_layer * l; a.k_b = (long)H * Scap * 64; a.k_h = (long)Scap * 64;
    a.v = m.xv + m.xkv_layer * l; a.v_b = (long)H * Scap * 64; a.v_h = (long)Scap * 64; a.v_blocked = 1;
    a.lim_row = nullptr; a.lim_seq = c->st.src_len; a.cap = Scap;
    LAUNCH(c, SPECDEC_KIND_GEMM_F32, st, sd::skinny2_head(st, bsrc, R, D, a, false, L.cwq, L.cbq, m.q, nullptr, nullptr, nullptr,
                                      nullptr, Lcap, L.cwo, P[pi ^ 1]));
    const sd::SkSrc csrc = with_sum(resolved(bsrc), P[pi ^ 1], H, L.cbo, L.ln2g, L.ln2b, S[si ^ 1]);
    if (l + 1 < m.d.dec_layers) {
      LAUNCH(c, SPECDEC_KIND_GEMM_BF16, st, sd::skinny2_ffn(st, csrc, R, D, L.w1, L.b1, F, L.w2, P[pi]));
      cur = with_sum(resolved(csrc), P[pi], sd::sk2_ffn_slices(F), L.b2, L.ln3g, L.ln3b, S[si]);
      si ^= 1;
      pi ^= 1;
    } else {
      LAUNCH(c, SPECDEC_KIND_GEMM_BF16, st, sd::skinny_proj(st, csrc, R, D, L.w1, F, L.b1, m.hid, true));
      LAUNCH(c, SPECDEC_KIND_GEMM_F32, st, sd::skinny_ffn2(st, resolved(csrc), R, D, m.hid, F, L.w2, L.b2, S[si]));
      cur = sd::SkSrc{2, S[si], L.ln3g, L.ln3b, nullptr, nullptr, nullptr, nullptr};
    }
  }
  *out = cur;
  return SPECDEC_OK;
}

// memory: [B][S_max][d] padded, or (packed) the model's own packed encoder rows (erow_b / epos / en_rows)
int cross_kv_from(specdec_ctx* c, Model& m, const bf16* memory, int B, int S_max, hipStream_t st, bool packed) {
  const int D = m.d.d_model;
  for (int l = 0; l < m.d.dec_layers; ++l)
    HIPCHK(c, sd::gemm_cross_kv(st, memory, m.dec[l].cwkv, B * S_max, D, D, m.dec[l].cbkv,
                                m.xk + m.xkv_layer * l, m.xv + m.xkv_layer * l, S_max, m.d.n_heads,
                                c->Scap, packed ? m.erow_b : nullptr, packed ? m.epos : nullptr,
                                packed ? m.en_rows : nullptr));
  if (m.kv8)   // whole arenas: every (layer, sequence of the batch limit, head, key row)
    HIPCHK(c, sd::quantize_cross_kv(st, m.xk, m.xv, (long)(m.xkv_layer / 64) * m.d.dec_layers, m.xk8, m.xv8, m.xks, m.xvs));
  m.has_memory = true;
  return SPECDEC_OK;
}

int check_ready(specdec_ctx* c, int role, bool need_memory) {
  if (!c) return SPECDEC_ERR_INVALID_ARG;
  if (role != SPECDEC_VERIFIER && role != SPECDEC_DRAFTER) return fail(c, SPECDEC_ERR_INVALID_ARG, "bad role %d", role);
  if (!c->state_bound) return fail(c, SPECDEC_ERR_BAD_STATE, "state buffer not bound");
  if (!c->m[role].bound) return fail(c, SPECDEC_ERR_BAD_STATE, "model of role %d not bound", role);
  if (c->B <= 0) return fail(c, SPECDEC_ERR_BAD_STATE, "specdec_begin not called");
  if (need_memory && !c->m[role].has_memory)
    return fail(c, SPECDEC_ERR_BAD_STATE, "no encoder memory: call specdec_encode or specdec_set_memory");
  return SPECDEC_OK;
}

}  // namespace

// ============================================================================= ABI
extern "C" {

int specdec_create(specdec_ctx** out, const specdec_limits* lim) {
  if (!out || !lim) return SPECDEC_ERR_INVALID_ARG;
  *out = nullptr;
  if (lim->max_batch < 1 || lim->max_batch > 4096 || lim->k_max < 1 || lim->k_max > 31 ||
      lim->max_src < 1 || lim->max_src > 65536 || lim->max_tgt < 1 || lim->max_tgt > 65536)
    return SPECDEC_ERR_INVALID_ARG;
  specdec_ctx* c = new (std::nothrow) specdec_ctx();
  if (!c) return SPECDEC_ERR_TOO_LARGE;
  c->lim = *lim;
  c->Tmax = 2 * lim->k_max + 1;
  c->Lcap = (lim->max_tgt + lim->k_max + 1 + 31) & ~31;   // rows of the KV arenas (32-key chunks)
  c->Scap = (lim->max_src + 31) & ~31;
  c->n_pos = c->Lcap > c->Scap ? c->Lcap : c->Scap;
  *out = c;
  return SPECDEC_OK;
}

void specdec_destroy(specdec_ctx* c) {
  if (!c) return;
  for (hipEvent_t e : c->prof_ev) (void)hipEventDestroy(e);
  delete c;
}

const char* specdec_last_error(const specdec_ctx* c) { return c ? c->err : "null context"; }

int specdec_configure(specdec_ctx* c, int32_t option, int32_t value) {
  if (!c) return SPECDEC_ERR_INVALID_ARG;
  if (value != 0 && value != 1) return fail(c, SPECDEC_ERR_INVALID_ARG, "option value %d (0 or 1)", value);
  switch (option) {
    case SPECDEC_OPT_SMALL_BATCH_KERNELS: c->no_skinny = (value == 0); break;
    case SPECDEC_OPT_LN_FOLD: c->no_ln_fold = (value == 0); break;
    case SPECDEC_OPT_RESIDENT: c->resident = (value == 1); break;
    case SPECDEC_OPT_SLICED_SUBLAYERS: c->sliced = (value == 1); break;
    case SPECDEC_OPT_FP8_WEIGHTS: c->fp8 = (value == 1); break;
    case SPECDEC_OPT_FP8_CROSS_KV: c->fp8_kv = (value == 1); break;
    case SPECDEC_OPT_WIDE_VOCAB_TILES: c->wide_vocab = (value == 1); break;
    default: return fail(c, SPECDEC_ERR_INVALID_ARG, "unknown option %d", option);
  }
  return SPECDEC_OK;
}

int specdec_num_weights(const specdec_model_desc* d, int32_t* out) {
  if (!out || !desc_ok(d)) return SPECDEC_ERR_INVALID_ARG;
  *out = n_weights(d);
  return SPECDEC_OK;
}

int specdec_weight_shape(const specdec_model_desc* d, int32_t idx, int64_t* rows, int64_t* cols) {
  if (!rows || !cols || !desc_ok(d) || idx < 0 || idx >= n_weights(d)) return SPECDEC_ERR_INVALID_ARG;
  weight_shape(d, idx, rows, cols);
  return SPECDEC_OK;
}

int specdec_state_bytes(const specdec_ctx* c, size_t* out) {
  if (!c || !out) return SPECDEC_ERR_INVALID_ARG;
  *out = carve_state(c, nullptr, nullptr);
  return SPECDEC_OK;
}

int specdec_bind_state(specdec_ctx* c, void* state, size_t bytes) {
  if (!c) return SPECDEC_ERR_INVALID_ARG;
  if (!state || (reinterpret_cast<uintptr_t>(state) & 255)) return fail(c, SPECDEC_ERR_INVALID_ARG, "state buffer null or not 256-byte aligned");
  if (bytes < carve_state(c, nullptr, nullptr)) return fail(c, SPECDEC_ERR_TOO_LARGE, "state buffer too small");
  carve_state(c, state, &c->st);
  c->state_bound = true;
  c->B = 0;
  return SPECDEC_OK;
}

int specdec_workspace_bytes(const specdec_ctx* c, const specdec_model_desc* d, size_t* out) {
  if (!c || !out) return SPECDEC_ERR_INVALID_ARG;
  if (!desc_ok(d)) return fail(c, SPECDEC_ERR_INVALID_ARG, "bad model description");
  *out = carve_model(c, d, nullptr, nullptr);
  return SPECDEC_OK;
}

int specdec_bind_model(specdec_ctx* c, specdec_role role, const specdec_model_desc* d, const void* const* weights,
                       int32_t nw, void* workspace, size_t bytes, void* stream) {
  if (!c) return SPECDEC_ERR_INVALID_ARG;
  if (role != SPECDEC_VERIFIER && role != SPECDEC_DRAFTER) return fail(c, SPECDEC_ERR_INVALID_ARG, "bad role");
  if (!desc_ok(d)) return fail(c, SPECDEC_ERR_INVALID_ARG, "bad model description (need d_model = 64*n_heads, d_ffn %% 64 == 0)");
  if (!weights || nw != n_weights(d)) return fail(c, SPECDEC_ERR_INVALID_ARG, "expected %d weight tensors, got %d", n_weights(d), nw);
  for (int i = 0; i < nw; ++i)
    if (!weights[i] || (reinterpret_cast<uintptr_t>(weights[i]) & 15))
      return fail(c, SPECDEC_ERR_INVALID_ARG, "weight %d null or not 16-byte aligned", i);
  if (!workspace || (reinterpret_cast<uintptr_t>(workspace) & 255)) return fail(c, SPECDEC_ERR_INVALID_ARG, "workspace null or not 256-byte aligned");
  if (bytes < carve_model(c, d, nullptr, nullptr)) return fail(c, SPECDEC_ERR_TOO_LARGE, "workspace too small");
  const Model& other = c->m[1 - role];
  if (other.bound && (other.d.vocab != d->vocab || other.d.bos_id != d->bos_id || other.d.eos_id != d->eos_id))
    return fail(c, SPECDEC_ERR_INVALID_ARG, "drafter and verifier must share the vocabulary and special ids");
  int dev_count = 0;
  if (hipGetDeviceCount(&dev_count) != hipSuccess || dev_count < 1) return fail(c, SPECDEC_ERR_NO_DEVICE, "no GPU");

  Model& m = c->m[role];
  m = Model();
  m.d = *d;
  auto W = [&](int i) { return static_cast<const bf16*>(weights[i]); };
  int i = 0;
  m.embed = W(i++);
  m.enc.resize(d->enc_layers);
  for (auto& L : m.enc) {
    L.wqkv = W(i++); L.bqkv = W(i++); L.wo = W(i++); L.bo = W(i++); L.ln1g = W(i++); L.ln1b = W(i++);
    L.w1 = W(i++); L.b1 = W(i++); L.w2 = W(i++); L.b2 = W(i++); L.ln2g = W(i++); L.ln2b = W(i++);
  }
  m.dec.resize(d->dec_layers);
  for (auto& L : m.dec) {
    L.wqkv = W(i++); L.bqkv = W(i++); L.wo = W(i++); L.bo = W(i++); L.ln1g = W(i++); L.ln1b = W(i++);
    L.cwq = W(i++); L.cbq = W(i++); L.cwkv = W(i++); L.cbkv = W(i++); L.cwo = W(i++); L.cbo = W(i++);
    L.ln2g = W(i++); L.ln2b = W(i++);
    L.w1 = W(i++); L.b1 = W(i++); L.w2 = W(i++); L.b2 = W(i++); L.ln3g = W(i++); L.ln3b = W(i++);
  }
  carve_model(c, d, workspace, &m);
  HIPCHK(c, sd::build_pos_table(S(stream), m.pe, c->n_pos, d->d_model));
  {
    const int D = d->d_model, F = d->d_ffn;
    float* f = m.fold;
    auto vec2 = [&](int n) { sd::LnFold o{f, f + n}; f += 2 * n; return o; };
    m.folds.resize(d->dec_layers);
    for (int l = 0; l < d->dec_layers; ++l) {
      const DecLayer& L = m.dec[l];
      LnFolds& o = m.folds[l];
      o.qkv = vec2(3 * D); o.cq = vec2(D); o.w1 = vec2(F);
      float* v = f;
      f += 9 * D;
      o.vo = v; o.vco = v + 3 * D; o.v2 = v + 6 * D;
      const bf16* g0 = l > 0 ? m.dec[l - 1].ln3g : nullptr;
      const bf16* b0 = l > 0 ? m.dec[l - 1].ln3b : nullptr;
      HIPCHK(c, sd::ln_sum_vecs(S(stream), L.bo, g0, b0, L.ln1g, D, v));
      HIPCHK(c, sd::ln_sum_vecs(S(stream), L.cbo, L.ln1g, L.ln1b, L.ln2g, D, v + 3 * D));
      HIPCHK(c, sd::ln_sum_vecs(S(stream), L.b2, L.ln2g, L.ln2b, L.ln3g, D, v + 6 * D));
      if (l > 0) HIPCHK(c, sd::ln_fold(S(stream), L.wqkv, m.dec[l - 1].ln3g, m.dec[l - 1].ln3b, L.bqkv, 3 * D, D, o.qkv));
      HIPCHK(c, sd::ln_fold(S(stream), L.cwq, L.ln1g, L.ln1b, L.cbq, D, D, o.cq));
      HIPCHK(c, sd::ln_fold(S(stream), L.w1, L.ln2g, L.ln2b, L.b1, F, D, o.w1));
    }
  }
  m.kv8 = c->fp8_kv;
  m.fp8 = c->fp8;
  if (m.fp8) {
    const int D = d->d_model, F = d->d_ffn;
    unsigned char* q = m.w8;
    float* sc = m.w8s;
    int rcq = SPECDEC_OK;
    auto quant = [&](const bf16* w, int N, int K) {
      sd::SkWeight o(q, sc);
      if (rcq == SPECDEC_OK && sd::quantize_rows_e4m3(S(stream), w, N, K, q, sc) != hipSuccess) rcq = SPECDEC_ERR_HIP;
      q += (size_t)N * K;
      sc += N;
      return o;
    };
    m.dec8.resize(d->dec_layers);
    for (int l = 0; l < d->dec_layers; ++l) {
      const DecLayer& L = m.dec[l];
      Fp8Layer& o = m.dec8[l];
      o.wqkv = quant(L.wqkv, 3 * D, D); o.wo = quant(L.wo, D, D);
      o.cwq = quant(L.cwq, D, D); o.cwo = quant(L.cwo, D, D);
      o.w1 = quant(L.w1, F, D); o.w2 = quant(L.w2, D, F);
    }
    m.embed8 = quant(m.embed, d->vocab, D);
    if (rcq != SPECDEC_OK) return fail(c, rcq, "FP8 weight quantisation failed: %s", hipGetErrorString(hipGetLastError()));
  }
  {
    std::vector<sd::RsLayer> rl(d->dec_layers);
    for (int l = 0; l < d->dec_layers; ++l) {
      const DecLayer& L = m.dec[l];
      rl[l] = sd::RsLayer{L.wqkv, L.bqkv, L.wo, L.bo, L.ln1g, L.ln1b, L.cwq, L.cbq, L.cwo, L.cbo, L.ln2g, L.ln2b,
                          L.w1, L.b1, L.w2, L.b2, L.ln3g, L.ln3b};
    }
    HIPCHK(c, hipMemcpy(m.rs_layers, rl.data(), rl.size() * sizeof(sd::RsLayer), hipMemcpyHostToDevice));
    HIPCHK(c, sd::fill_i32(S(stream), reinterpret_cast<int*>(m.rs_bar), 0, sd::kRsBarWords));
    m.rs_parity = 0;
  }
  m.bound = true;
  return SPECDEC_OK;
}

int specdec_begin(specdec_ctx* c, int32_t B, int32_t max_new, void* stream) {
  if (!c) return SPECDEC_ERR_INVALID_ARG;
  if (!c->state_bound) return fail(c, SPECDEC_ERR_BAD_STATE, "state buffer not bound");
  if (!c->m[0].bound && !c->m[1].bound) return fail(c, SPECDEC_ERR_BAD_STATE, "no model bound");
  if (B < 1 || max_new < 0) return fail(c, SPECDEC_ERR_INVALID_ARG, "B = %d, max_new = %d", B, max_new);
  if (B > c->lim.max_batch) return fail(c, SPECDEC_ERR_TOO_LARGE, "B = %d exceeds max_batch = %d", B, c->lim.max_batch);
  const Model& any = c->m[0].bound ? c->m[0] : c->m[1];
  if (max_new > c->lim.max_tgt) max_new = c->lim.max_tgt;   // no stream grows beyond the arena
  HIPCHK(c, sd::begin_state(S(stream), c->st, B, max_new, c->lim.max_tgt, any.d.bos_id));
  if (c->m[0].bound) {   // a new run clears the resident kernel's counters and error flag
    HIPCHK(c, sd::fill_i32(S(stream), reinterpret_cast<int*>(c->m[0].rs_bar), 0, sd::kRsBarWords));
    c->m[0].rs_parity = 0;
  }
  c->B = B;
  c->max_new = max_new;
  c->last_T = 0;
  c->last_k_draft = 0;
  c->uncached_ub[0] = 0;
  c->uncached_ub[1] = 1;
  c->trusted[0] = c->trusted[1] = false;
  c->m[0].has_memory = c->m[1].has_memory = false;
  return SPECDEC_OK;
}

int specdec_set_memory(specdec_ctx* c, specdec_role role, const void* memory, const int32_t* src_len,
                       int32_t S_max, void* stream) {
  int rc = check_ready(c, role, false);
  if (rc) return rc;
  if (!memory || !src_len || (reinterpret_cast<uintptr_t>(memory) & 15)) return fail(c, SPECDEC_ERR_INVALID_ARG, "memory/src_len null or misaligned");
  if (S_max < 1) return fail(c, SPECDEC_ERR_INVALID_ARG, "S_max = %d", S_max);
  if (S_max > c->lim.max_src) return fail(c, SPECDEC_ERR_TOO_LARGE, "S_max = %d exceeds max_src = %d", S_max, c->lim.max_src);
  HIPCHK(c, sd::set_src_len(S(stream), c->st, src_len, c->B, S_max));
  c->S_cur = S_max;
  c->m[role].enc_packed = false;
  return cross_kv_from(c, c->m[role], static_cast<const bf16*>(memory), c->B, S_max, S(stream), false);
}

// Encoder of one model over the sources' rows without padding (sequence b owns rows erow_start[b] ..
// + src_len[b] - 1; grids are sized for B*S_max rows, row tiles beyond the real count return at once);
// leaves the memory (bf16, packed) in m.exb.
static int encoder_pass(specdec_ctx* c, Model& m, const int32_t* src, int B, int S_max, hipStream_t st) {
  const int R = B * S_max, D = m.d.d_model, F = m.d.d_ffn, H = m.d.n_heads, Scap = c->Scap;
  const size_t Re = (size_t)c->lim.max_batch * Scap;
  bf16* eq = m.eqkv;                 // [R][d]
  bf16* ek = m.eqkv + Re * D;        // [B][H][Scap][64]
  bf16* ev = m.eqkv + 2 * Re * D;    // [B][H][Scap/8][64][8]
  const int* nr = m.en_rows;
  HIPCHK(c, sd::encoder_rows_packed(st, src, c->st.src_len, m.etok, m.epos, m.erow_b, m.erow_start, m.en_rows, B, S_max,
                                    m.d.vocab));
  LAUNCH(c, SPECDEC_KIND_OTHER, st, sd::embed_rows(st, m.etok, m.epos, m.embed, m.pe, m.ex, m.exb, R, D));
  for (int l = 0; l < m.d.enc_layers; ++l) {
    const EncLayer& L = m.enc[l];
    LAUNCH(c, SPECDEC_KIND_GEMM_QKV, st, sd::gemm_enc_qkv(st, m.exb, L.wqkv, R, D, D, L.bqkv, eq, ek, ev, S_max, H, Scap,
                                                          m.erow_b, m.epos, nr));
    sd::AttnArgs a{};
    a.q = eq; a.q_b = (long)S_max * D; a.q_row = D;
    a.k = ek; a.k_b = (long)H * Scap * 64; a.k_h = (long)Scap * 64; a.k_row = 64;
    a.v = ev; a.v_b = (long)H * Scap * 64; a.v_h = (long)Scap * 64; a.v_row = 64; a.v_blocked = 1;
    a.o = m.eatt; a.o_b = (long)S_max * D; a.o_row = D;
    a.q_count = c->st.src_len; a.q_off = m.erow_start; a.lim_row = nullptr; a.lim_seq = c->st.src_len;
    a.T = S_max; a.H = H; a.B = B;
    a.key_split = S_max > 256; a.cap = Scap;
    LAUNCH(c, SPECDEC_KIND_ATTN, st, sd::attention(st, a));
    LAUNCH(c, SPECDEC_KIND_GEMM_F32, st, sd::gemm_f32(st, m.eatt, D, L.wo, R, D, D, L.bo, m.ex, m.ex, D, nr));
    LAUNCH(c, SPECDEC_KIND_LN, st, sd::layer_norm(st, m.ex, L.ln1g, L.ln1b, m.exb, R, D, nr));
    LAUNCH(c, SPECDEC_KIND_GEMM_BF16, st, sd::gemm_bf16(st, m.exb, D, L.w1, R, F, D, L.b1, m.ehid, F, true, nr));
    LAUNCH(c, SPECDEC_KIND_GEMM_F32, st, sd::gemm_f32(st, m.ehid, F, L.w2, R, D, F, L.b2, m.ex, m.ex, D, nr));
    LAUNCH(c, SPECDEC_KIND_LN, st, sd::layer_norm(st, m.ex, L.ln2g, L.ln2b, m.exb, R, D, nr));
  }
  m.enc_packed = true;
  return SPECDEC_OK;
}

int specdec_encode(specdec_ctx* c, const int32_t* src, const int32_t* src_len, int32_t S_max, void* stream) {
  if (!c) return SPECDEC_ERR_INVALID_ARG;
  if (!c->state_bound || c->B <= 0) return fail(c, SPECDEC_ERR_BAD_STATE, "bind state and call specdec_begin first");
  if (!src || !src_len) return fail(c, SPECDEC_ERR_INVALID_ARG, "null src/src_len");
  if (S_max < 1) return fail(c, SPECDEC_ERR_INVALID_ARG, "S_max = %d", S_max);
  if (S_max > c->lim.max_src) return fail(c, SPECDEC_ERR_TOO_LARGE, "S_max = %d exceeds max_src = %d", S_max, c->lim.max_src);
  int n = 0;
  for (int r = 0; r < 2; ++r) n += (c->m[r].bound && c->m[r].d.enc_layers > 0) ? 1 : 0;
  if (n == 0) return fail(c, SPECDEC_ERR_BAD_STATE, "no bound model has an encoder");
  hipStream_t st = S(stream);
  HIPCHK(c, sd::set_src_len(st, c->st, src_len, c->B, S_max));
  c->S_cur = S_max;
  for (int r = 0; r < 2; ++r) {
    Model& m = c->m[r];
    if (!m.bound || m.d.enc_layers == 0) continue;
    int rc = encoder_pass(c, m, src, c->B, S_max, st);
    if (rc) return rc;
    rc = cross_kv_from(c, m, m.exb, c->B, S_max, st, true);
    if (rc) return rc;
  }
  return SPECDEC_OK;
}

int specdec_set_stream(specdec_ctx* c, const int32_t* tokens, const int32_t* len, int32_t L_max, void* stream) {
  if (!c) return SPECDEC_ERR_INVALID_ARG;
  if (!c->state_bound || c->B <= 0) return fail(c, SPECDEC_ERR_BAD_STATE, "bind state and call specdec_begin first");
  if (!tokens || !len) return fail(c, SPECDEC_ERR_INVALID_ARG, "null tokens/len");
  if (L_max < 0) return fail(c, SPECDEC_ERR_INVALID_ARG, "L_max = %d", L_max);
  if (L_max > c->lim.max_tgt) return fail(c, SPECDEC_ERR_TOO_LARGE, "L_max = %d exceeds max_tgt = %d", L_max, c->lim.max_tgt);
  HIPCHK(c, sd::set_stream(S(stream), c->st, tokens, len, c->B, L_max, c->max_new, c->lim.max_tgt));
  c->uncached_ub[0] = L_max;
  c->uncached_ub[1] = L_max + 1;
  c->trusted[0] = c->trusted[1] = false;
  c->last_T = 0;
  return SPECDEC_OK;
}

int specdec_load_cache(specdec_ctx* c, specdec_role role, const void* k_cache, const void* v_cache,
                       const int32_t* n, int32_t L_max, void* stream) {
  int rc = check_ready(c, role, false);
  if (rc) return rc;
  if (!k_cache || !v_cache || !n) return fail(c, SPECDEC_ERR_INVALID_ARG, "null cache/n");
  if ((reinterpret_cast<uintptr_t>(k_cache) | reinterpret_cast<uintptr_t>(v_cache)) & 15) return fail(c, SPECDEC_ERR_INVALID_ARG, "cache not 16-byte aligned");
  if (L_max < 0) return fail(c, SPECDEC_ERR_INVALID_ARG, "L_max = %d", L_max);
  if (L_max > c->lim.max_tgt + 1) return fail(c, SPECDEC_ERR_TOO_LARGE, "L_max = %d exceeds max_tgt + 1", L_max);
  Model& m = c->m[role];
  const int H = m.d.n_heads;
  const size_t flat_layer = (size_t)c->B * L_max * m.d.d_model;
  for (int l = 0; l < m.d.dec_layers; ++l) {
    HIPCHK(c, sd::cache_from_flat(S(stream), m.kc + m.kv_layer * l, static_cast<const bf16*>(k_cache) + flat_layer * l, c->B, H, c->Lcap, L_max, false));
    HIPCHK(c, sd::cache_from_flat(S(stream), m.vc + m.kv_layer * l, static_cast<const bf16*>(v_cache) + flat_layer * l, c->B, H, c->Lcap, L_max, false));
  }
  HIPCHK(c, sd::set_cached(S(stream), c->st, role, n, c->B, L_max));
  c->trusted[role] = true;
  return SPECDEC_OK;
}

int specdec_set_prefix(specdec_ctx* c, specdec_role role, const int32_t* tokens, const int32_t* len, int32_t L_max,
                       const void* k_cache, const void* v_cache, void* stream) {
  int rc = check_ready(c, role, false);
  if (rc) return rc;
  if (!k_cache || !v_cache) return fail(c, SPECDEC_ERR_INVALID_ARG, "null cache");
  rc = specdec_set_stream(c, tokens, len, L_max, stream);
  if (rc) return rc;
  // every position below j is cached (the drafter's own count of u_j is left to its next pass)
  return specdec_load_cache(c, role, k_cache, v_cache, len, L_max, stream);
}

int specdec_prefill(specdec_ctx* c, specdec_role role, void* stream) {
  int rc = check_ready(c, role, true);
  if (rc) return rc;
  Model& m = c->m[role];
  hipStream_t st = S(stream);
  const int T = c->Tmax;
  while (c->uncached_ub[role] > 0) {
    LAUNCH(c, SPECDEC_KIND_OTHER, st, sd::assemble_embed_stream(st, c->st, m.rm, role, c->B, T, 0, m.d.mask_id, m.d.pad_id, m.d.vocab,
                                        m.new_rows, m.embed, m.pe, m.x, m.xb, m.d.d_model, false));
    rc = decoder_layers(c, m, c->B, T, st, true);
    if (rc) return rc;
    HIPCHK(c, sd::advance_cached(st, c->st, role, m.new_rows, c->B));
    c->uncached_ub[role] -= T;
  }
  c->uncached_ub[role] = 0;
  c->trusted[role] = false;
  return SPECDEC_OK;
}

int specdec_draft(specdec_ctx* c, int32_t k, int32_t* draft, float* logits, void* stream) {
  int rc = check_ready(c, SPECDEC_DRAFTER, true);
  if (rc) return rc;
  if (!draft) return fail(c, SPECDEC_ERR_INVALID_ARG, "null draft");
  if (k < 1) return fail(c, SPECDEC_ERR_INVALID_ARG, "k = %d", k);
  if (k > c->lim.k_max) return fail(c, SPECDEC_ERR_TOO_LARGE, "k = %d exceeds k_max = %d", k, c->lim.k_max);
  Model& m = c->m[SPECDEC_DRAFTER];
  hipStream_t st = S(stream);
  // stream tokens the drafter has not ingested yet: at most k_max + 1 fit beside the k slots
  int ub = c->trusted[1] ? 1 : c->uncached_ub[1];
  if (ub < 1) ub = 1;
  if (ub > c->lim.k_max + 1) {
    rc = specdec_prefill(c, SPECDEC_DRAFTER, stream);
    if (rc) return rc;
    ub = 1;
  }
  const int B = c->B, T = ub + k;
  // rows packed sequence after sequence: a sequence brings 1 .. k_max + 1 new stream rows, the
  // grids are sized for the most (the GEMMs with LayerNorm folded in know how to stop early)
  const bool packed = !c->no_ln_fold;
  LAUNCH(c, SPECDEC_KIND_OTHER, st, sd::assemble_embed_stream(st, c->st, m.rm, SPECDEC_DRAFTER, B, T, k, m.d.mask_id, m.d.pad_id,
                                      m.d.vocab, m.new_rows, m.embed, m.pe, m.x, m.xb, m.d.d_model, packed));
  rc = decoder_layers(c, m, B, T, st, true, k, packed);
  if (rc) return rc;
  const int R = B * k, tc = sd::vocab_tile_cols(R), n_tiles = (m.d.vocab + tc - 1) / tc;
  LAUNCH(c, SPECDEC_KIND_VOCAB, st, sd::vocab_stats(st, m.slots, m.embed, R, m.d.vocab, m.d.d_model, nullptr, nullptr, m.part, logits, c->wide_vocab));
  LAUNCH(c, SPECDEC_KIND_ACCEPT, st, sd::merge_drafts(st, m.part, n_tiles, m.row_stats, c->st, B, k, m.d.pad_id, m.new_rows,
                                      m.rm.seq_rows, draft));
  c->uncached_ub[1] = 0;
  c->trusted[1] = false;
  c->last_k_draft = k;
  return SPECDEC_OK;
}

}  // extern "C"

// Scratch of specdec_verify_static (callers that may not allocate or bring a workspace for it):
// vocabulary partial records, draft logits and merged row statistics of one verification pass.
// One array per GPU, held until the process ends and shared by every call on that GPU.  In host
// code the name is only a handle for hipGetSymbolAddress; kernels get the device address.
constexpr size_t kStaticRows = 1408;                                   // B * (k + 1) of the largest pass it serves
constexpr size_t kStaticPartFloats = kStaticRows * 256 * sd::kPartF;   // rows x tiles x record (5.5 MiB)
constexpr size_t kStaticFloats = kStaticPartFloats + kStaticRows + kStaticRows * sd::kRowStats;
static __device__ __align__(256) float scratch[kStaticFloats];

namespace {

// Scratch of a verification pass; specdec_verify carves it from the caller's workspace.
struct VerifyScratch {
  float *part, *zd, *row_stats;
};
constexpr int kMaxDevices = 64;
float* scratch_ptr[kMaxDevices] = {nullptr};                  // device address of `scratch` on each GPU

int verify_impl(specdec_ctx* c, const int32_t* draft, int32_t k, int32_t beta, float tau, int32_t* accept_len,
                int32_t* next_token, float* logits, void* stream, const VerifyScratch* ext) {
  int rc = check_ready(c, SPECDEC_VERIFIER, true);
  if (rc) return rc;
  if (!accept_len || !next_token || (!draft && k > 0)) return fail(c, SPECDEC_ERR_INVALID_ARG, "null draft/accept_len/next_token");
  if (k < 0) return fail(c, SPECDEC_ERR_INVALID_ARG, "k = %d", k);
  if (k > c->lim.k_max) return fail(c, SPECDEC_ERR_TOO_LARGE, "k = %d exceeds k_max = %d", k, c->lim.k_max);
  Model& m = c->m[SPECDEC_VERIFIER];
  if (beta < 1 || beta > m.d.vocab) return fail(c, SPECDEC_ERR_INVALID_ARG, "beta = %d outside [1, vocab]", beta);
  if (!(tau >= 0.f) || !std::isfinite(tau)) return fail(c, SPECDEC_ERR_INVALID_ARG, "tau must be finite and >= 0");
  if (c->uncached_ub[0] > 0 && !c->trusted[0]) return fail(c, SPECDEC_ERR_BAD_STATE, "verifier cache does not cover the stream: call specdec_prefill or specdec_load_cache");
  hipStream_t st = S(stream);
  const int B = c->B, T = k + 1, R = B * T;
  const bool small = skinny_ok(c, m, R, T);   // the small-batch kernels embed the rows themselves
  VerifyScratch vs{m.part, m.zd, m.row_stats};
  if (ext) {
    const size_t tiles = small ? (m.d.vocab + 63) / 64 : (m.d.vocab + sd::vocab_tile_cols(R) - 1) / sd::vocab_tile_cols(R);
    if ((size_t)R > kStaticRows || (size_t)R * tiles * sd::kPartF > kStaticPartFloats)
      return fail(c, SPECDEC_ERR_TOO_LARGE, "pass of %d rows x %zu vocabulary tiles exceeds the static scratch "
                  "(%zu rows, %zu floats of records)", R, tiles, kStaticRows, kStaticPartFloats);
    vs = *ext;
  }
  if (small)
    LAUNCH(c, SPECDEC_KIND_OTHER, st, sd::assemble_verify(st, c->st, m.rm, draft, B, k, m.d.vocab));
  else
    LAUNCH(c, SPECDEC_KIND_OTHER, st, sd::assemble_embed_verify(st, c->st, m.rm, draft, B, k, m.d.vocab, m.embed, m.pe, m.x, m.xb,
                                        m.d.d_model));
  const unsigned* failed = nullptr;
  int n_tiles = (m.d.vocab + 63) / 64;   // per-row partial records of the vocabulary kernel that ran
  if (small && (m.fp8 || m.kv8) && (c->resident || c->sliced))
    return fail(c, SPECDEC_ERR_BAD_STATE, "a model bound with FP8 weights or FP8 cross keys/values runs small passes on the default kernels only");
  if (small && c->resident) {
    sd::RsArgs a{};
    a.R = R; a.T = T; a.B = B; a.H = m.d.n_heads; a.V = m.d.vocab; a.Lcap = c->Lcap; a.Scap = c->Scap;
    a.n_layers = m.d.dec_layers; a.layers = m.rs_layers;
    a.row_tok = m.rm.row_tok; a.row_pos = m.rm.row_pos; a.row_b = m.rm.row_b; a.row_lim = m.rm.row_lim;
    a.row_draft = m.rm.row_draft; a.seq_rows = m.rm.seq_rows; a.src_len = c->st.src_len;
    a.E = m.embed; a.pe = m.pe; a.xs0 = m.x; a.xs1 = m.x2; a.q = m.q; a.hid = m.hid;
    a.kc = m.kc; a.vc = m.vc; a.xk = m.xk; a.xv = m.xv; a.kv_layer = m.kv_layer; a.xkv_layer = m.xkv_layer;
    a.zd = vs.zd; a.part = vs.part; a.logits = logits;
    a.bar = m.rs_bar; a.parity = m.rs_parity;
    m.rs_seq = m.rs_seq >= 0x3fffffff ? 1 : m.rs_seq + 1;
    a.seq = m.rs_seq;
    m.rs_parity ^= 1;
    LAUNCH(c, SPECDEC_KIND_RESIDENT, st, sd::resident_verify(st, a, m.d.d_model, m.d.d_ffn));
    failed = m.rs_bar + 16;
    c->fin_x = nullptr;   // (the resident kernel keeps its last sum to itself)
  } else if (small) {
    sd::SkSrc fin{};
    if (c->sliced && sd::sk2_supported(m.d.d_model, m.d.d_ffn) && m.d.n_heads <= sd::kSk2MaxParts)
      rc = decoder_layers_sliced(c, m, B, T, st, &fin);
    else
      rc = decoder_layers_skinny(c, m, B, T, st, &fin);
    if (rc) return rc;
    LAUNCH(c, SPECDEC_KIND_VOCAB, st, sd::skinny_vocab(st, fin, R, m.d.d_model, m.fp8 ? m.embed8 : sd::SkWeight(m.embed), m.d.vocab, m.rm.row_draft, vs.zd, vs.part, logits));
    c->fin_x = fin.xs; c->fin_g = fin.g; c->fin_b = fin.b;
  } else {
    rc = decoder_layers(c, m, B, T, st, true);
    if (rc) return rc;
    c->fin_x = m.x; c->fin_g = nullptr; c->fin_b = nullptr;   // normalised in place by the last LayerNorm
    n_tiles = (m.d.vocab + sd::vocab_tile_cols(R) - 1) / sd::vocab_tile_cols(R);
    LAUNCH(c, SPECDEC_KIND_VOCAB, st, sd::vocab_stats(st, m.xb, m.embed, R, m.d.vocab, m.d.d_model, m.rm.row_draft, vs.zd, vs.part, logits, c->wide_vocab));
  }
  LAUNCH(c, SPECDEC_KIND_ACCEPT, st, sd::merge_accept(st, vs.part, vs.zd, n_tiles, vs.row_stats, c->st, B, k, beta, tau, m.d.pad_id,
                                      accept_len, next_token, failed));
  c->last_T = k + 1;
  c->last_row_stats = vs.row_stats;
  return SPECDEC_OK;
}

}  // namespace

extern "C" {

int specdec_verify(specdec_ctx* c, const int32_t* draft, int32_t k, int32_t beta, float tau, int32_t* accept_len,
                   int32_t* next_token, float* logits, void* stream) {
  return verify_impl(c, draft, k, beta, tau, accept_len, next_token, logits, stream, nullptr);
}

int specdec_verify_static(specdec_ctx* c, const int32_t* draft, int32_t k, int32_t beta, float tau, int32_t* accept_len,
                          int32_t* next_token, float* logits, void* stream) {
  if (!c) return SPECDEC_ERR_INVALID_ARG;
  const int ready = check_ready(c, SPECDEC_VERIFIER, true);   // call-order errors before the device is touched
  if (ready) return ready;
  int dev = -1;
  HIPCHK(c, hipGetDevice(&dev));
  if (dev < 0 || dev >= kMaxDevices) return fail(c, SPECDEC_ERR_HIP, "device ordinal %d out of range", dev);
  if (!scratch_ptr[dev]) {   // once per GPU, with that GPU current: each GPU holds its own copy of the array
    float* p = nullptr;
    HIPCHK(c, hipGetSymbolAddress(reinterpret_cast<void**>(&p), HIP_SYMBOL(scratch)));
    if (!p) return fail(c, SPECDEC_ERR_HIP, "hipGetSymbolAddress returned a null address");
    scratch_ptr[dev] = p;
  }
  float* base = scratch_ptr[dev];
  const VerifyScratch vs{base, base + kStaticPartFloats, base + kStaticPartFloats + kStaticRows};
  return verify_impl(c, draft, k, beta, tau, accept_len, next_token, logits, stream, &vs);
}

int specdec_bind_draft_heads(specdec_ctx* c, int32_t n_heads, const void* w1, const void* b1, const void* w2,
                             const void* b2) {
  if (!c) return SPECDEC_ERR_INVALID_ARG;
  if (!c->m[0].bound) return fail(c, SPECDEC_ERR_BAD_STATE, "bind the verifier first: the heads sit on top of it");
  if (n_heads < 1) return fail(c, SPECDEC_ERR_INVALID_ARG, "n_heads = %d", n_heads);
  if (n_heads > c->lim.k_max) return fail(c, SPECDEC_ERR_TOO_LARGE, "n_heads = %d exceeds k_max = %d", n_heads, c->lim.k_max);
  if (!w1 || !b1 || !w2 || !b2) return fail(c, SPECDEC_ERR_INVALID_ARG, "null head weights");
  if ((reinterpret_cast<uintptr_t>(w1) | reinterpret_cast<uintptr_t>(b1) | reinterpret_cast<uintptr_t>(w2) |
       reinterpret_cast<uintptr_t>(b2)) & 15)
    return fail(c, SPECDEC_ERR_INVALID_ARG, "head weights not 16-byte aligned");
  c->n_draft_heads = n_heads;
  c->hw1 = static_cast<const bf16*>(w1); c->hb1 = static_cast<const bf16*>(b1);
  c->hw2 = static_cast<const bf16*>(w2); c->hb2 = static_cast<const bf16*>(b2);
  return SPECDEC_OK;
}

int specdec_draft_heads(specdec_ctx* c, const int32_t* accept_len, int32_t k, int32_t* draft, float* logits, void* stream) {
  int rc = check_ready(c, SPECDEC_VERIFIER, false);
  if (rc) return rc;
  if (!accept_len || !draft) return fail(c, SPECDEC_ERR_INVALID_ARG, "null accept_len/draft");
  if (c->n_draft_heads < 1) return fail(c, SPECDEC_ERR_BAD_STATE, "no drafting heads bound");
  if (k < 1) return fail(c, SPECDEC_ERR_INVALID_ARG, "k = %d", k);
  if (k > c->n_draft_heads) return fail(c, SPECDEC_ERR_TOO_LARGE, "k = %d exceeds the %d heads bound", k, c->n_draft_heads);
  if (c->last_T <= 0) return fail(c, SPECDEC_ERR_BAD_STATE, "specdec_draft_heads needs the hidden states of a specdec_verify "
                                  "(call it after specdec_verify, before specdec_commit)");
  if (!c->fin_x) return fail(c, SPECDEC_ERR_BAD_STATE, "the latest verification pass (resident kernel) kept no hidden states");
  Model& m = c->m[SPECDEC_VERIFIER];
  hipStream_t st = S(stream);
  const int B = c->B, D = m.d.d_model, F = m.d.d_ffn, nh = c->n_draft_heads, R = B * k;
  // the verifier's final hidden state at each sequence's bifurcation row -> bf16 [B][d], fp32 x k
  LAUNCH(c, SPECDEC_KIND_OTHER, st, sd::head_rows(st, c->fin_x, c->fin_g, c->fin_b, accept_len, B, c->last_T, k, D, m.att, m.hx));
  // first layer of the k heads in one product: hid [B][k*F] = ReLU(h W1_all^T + b1_all)
  LAUNCH(c, SPECDEC_KIND_GEMM_BF16, st, sd::gemm_bf16(st, m.att, D, c->hw1, B, k * F, D, c->hb1, m.hid, k * F, true));
  // second layer, head by head (block diagonal): row b*k + i of hx += hid[b][i*F .. ] W2_i^T + b2_i
  for (int i = 0; i < k; ++i)
    LAUNCH(c, SPECDEC_KIND_GEMM_F32, st, sd::gemm_f32(st, m.hid + (size_t)i * F, k * F, c->hw2 + (size_t)i * D * F, B, D, F,
                                     c->hb2 + (size_t)i * D, m.hx + (size_t)i * D, m.hx + (size_t)i * D, k * D));
  HIPCHK(c, sd::f32_to_bf16(st, m.hx, m.slots, (long)R * D));
  const int tc = sd::vocab_tile_cols(R), n_tiles = (m.d.vocab + tc - 1) / tc;
  LAUNCH(c, SPECDEC_KIND_VOCAB, st, sd::vocab_stats(st, m.slots, m.embed, R, m.d.vocab, D, nullptr, nullptr, m.part, logits, c->wide_vocab));
  LAUNCH(c, SPECDEC_KIND_ACCEPT, st, sd::merge_head_drafts(st, m.part, n_tiles, m.row_stats, c->st, accept_len, B, k, m.d.pad_id, draft));
  (void)nh;
  return SPECDEC_OK;
}

int specdec_commit(specdec_ctx* c, const int32_t* accept_len, const int32_t* next_token, int32_t* n_active, void* stream) {
  int rc = check_ready(c, SPECDEC_VERIFIER, false);
  if (rc) return rc;
  if (!accept_len || !next_token) return fail(c, SPECDEC_ERR_INVALID_ARG, "null accept_len/next_token");
  if (c->last_T <= 0) return fail(c, SPECDEC_ERR_BAD_STATE, "specdec_commit without a preceding specdec_verify");
  HIPCHK(c, sd::commit_rows(S(stream), c->st, accept_len, next_token, c->B, c->last_T - 1, c->m[0].d.eos_id, n_active));
  c->last_T = 0;
  c->uncached_ub[1] += c->lim.k_max + 1;
  return SPECDEC_OK;
}

int specdec_rewind(specdec_ctx* c, const int32_t* len, void* stream) {
  if (!c) return SPECDEC_ERR_INVALID_ARG;
  if (!c->state_bound || c->B <= 0) return fail(c, SPECDEC_ERR_BAD_STATE, "begin not called");
  if (!len) return fail(c, SPECDEC_ERR_INVALID_ARG, "null len");
  HIPCHK(c, sd::rewind_state(S(stream), c->st, len, c->B));
  c->last_T = 0;
  return SPECDEC_OK;
}

int specdec_profile_select(specdec_ctx* c, int32_t kind) {
  if (!c) return SPECDEC_ERR_INVALID_ARG;
  if (kind < SPECDEC_KIND_NONE || kind >= SPECDEC_KIND_COUNT) return fail(c, SPECDEC_ERR_INVALID_ARG, "bad kernel kind %d", kind);
  if (kind != SPECDEC_KIND_NONE && c->prof_ev.empty()) {
    c->prof_ev.reserve(2 * kProfPairs);
    for (int i = 0; i < 2 * kProfPairs; ++i) {
      hipEvent_t e;
      HIPCHK(c, hipEventCreate(&e));
      c->prof_ev.push_back(e);
    }
  }
  c->prof_kind = kind;
  c->prof_used = 0;
  return SPECDEC_OK;
}

int specdec_profile_read(specdec_ctx* c, double* total_ms, int32_t* launches) {
  if (!c || !total_ms || !launches) return SPECDEC_ERR_INVALID_ARG;
  double tot = 0.0;
  for (int i = 0; i + 1 < c->prof_used; i += 2) {
    HIPCHK(c, hipEventSynchronize(c->prof_ev[i + 1]));
    float ms = 0.f;
    HIPCHK(c, hipEventElapsedTime(&ms, c->prof_ev[i], c->prof_ev[i + 1]));
    tot += ms;
  }
  *total_ms = tot;
  *launches = c->prof_used / 2;
  c->prof_used = 0;
  return SPECDEC_OK;
}

int specdec_get_output(specdec_ctx* c, int32_t* tokens, int32_t out_cap, int32_t* out_len, int32_t* finished, void* stream) {
  if (!c) return SPECDEC_ERR_INVALID_ARG;
  if (!c->state_bound || c->B <= 0) return fail(c, SPECDEC_ERR_BAD_STATE, "nothing to read: begin not called");
  if (!tokens || !out_len || out_cap < 1) return fail(c, SPECDEC_ERR_INVALID_ARG, "null output or out_cap < 1");
  const Model& any = c->m[0].bound ? c->m[0] : c->m[1];
  HIPCHK(c, sd::get_output(S(stream), c->st, tokens, out_cap, out_len, finished, c->B, any.d.pad_id));
  return SPECDEC_OK;
}

int specdec_get_cache(specdec_ctx* c, specdec_role role, void* k_cache, void* v_cache, int32_t L, void* stream) {
  int rc = check_ready(c, role, false);
  if (rc) return rc;
  if (!k_cache || !v_cache) return fail(c, SPECDEC_ERR_INVALID_ARG, "null cache");
  if (L < 1 || L > c->Lcap) return fail(c, SPECDEC_ERR_INVALID_ARG, "L = %d outside [1, %d]", L, c->Lcap);
  Model& m = c->m[role];
  const size_t flat_layer = (size_t)c->B * L * m.d.d_model;
  for (int l = 0; l < m.d.dec_layers; ++l) {
    HIPCHK(c, sd::cache_to_flat(S(stream), m.kc + m.kv_layer * l, static_cast<bf16*>(k_cache) + flat_layer * l, c->B, m.d.n_heads, c->Lcap, L, false));
    HIPCHK(c, sd::cache_to_flat(S(stream), m.vc + m.kv_layer * l, static_cast<bf16*>(v_cache) + flat_layer * l, c->B, m.d.n_heads, c->Lcap, L, false));
  }
  return SPECDEC_OK;
}

int specdec_get_memory(specdec_ctx* c, specdec_role role, void* memory, void* stream) {
  int rc = check_ready(c, role, true);
  if (rc) return rc;
  if (!memory) return fail(c, SPECDEC_ERR_INVALID_ARG, "null memory");
  Model& m = c->m[role];
  if (m.d.enc_layers == 0 || !m.exb) return fail(c, SPECDEC_ERR_BAD_STATE, "model has no encoder");
  if (!m.enc_packed) return fail(c, SPECDEC_ERR_BAD_STATE, "the memory in use was supplied by specdec_set_memory, not computed by specdec_encode");
  HIPCHK(c, sd::unpack_rows(S(stream), m.exb, m.erow_start, c->st.src_len, static_cast<bf16*>(memory), c->B, c->S_cur,
                            m.d.d_model));
  return SPECDEC_OK;
}

int specdec_get_draft_stats(specdec_ctx* c, float* stats, void* stream) {
  int rc = check_ready(c, SPECDEC_DRAFTER, false);
  if (rc) return rc;
  if (!stats) return fail(c, SPECDEC_ERR_INVALID_ARG, "null stats");
  if (c->last_k_draft <= 0) return fail(c, SPECDEC_ERR_BAD_STATE, "no drafter pass to report");
  const size_t n = (size_t)c->B * c->last_k_draft * SPECDEC_ROW_STATS;
  HIPCHK(c, hipMemcpyAsync(stats, c->m[1].row_stats, n * sizeof(float), hipMemcpyDeviceToDevice, S(stream)));
  return SPECDEC_OK;
}

int specdec_get_counters(specdec_ctx* c, int32_t* counters, void* stream) {
  if (!c) return SPECDEC_ERR_INVALID_ARG;
  if (!c->state_bound || c->B <= 0) return fail(c, SPECDEC_ERR_BAD_STATE, "begin not called");
  if (!counters) return fail(c, SPECDEC_ERR_INVALID_ARG, "null counters");
  HIPCHK(c, hipMemcpyAsync(counters, c->st.scratch, SPECDEC_COUNTERS * sizeof(int32_t), hipMemcpyDeviceToDevice, S(stream)));
  return SPECDEC_OK;
}

int specdec_quantize_rows(specdec_ctx* c, const void* w, int64_t N, int64_t K, void* codes, float* scale,
                               void* stream) {
  if (!c) return SPECDEC_ERR_INVALID_ARG;
  if (!w || !codes || !scale) return fail(c, SPECDEC_ERR_INVALID_ARG, "null w/codes/scale");
  if (N < 0 || K <= 0 || K % 8 != 0 || N > INT32_MAX || K > INT32_MAX)
    return fail(c, SPECDEC_ERR_INVALID_ARG, "N = %lld, K = %lld (K must be a positive multiple of 8)", (long long)N, (long long)K);
  if ((reinterpret_cast<uintptr_t>(w) & 15) || (reinterpret_cast<uintptr_t>(codes) & 7))
    return fail(c, SPECDEC_ERR_INVALID_ARG, "w must be 16-byte aligned, codes 8-byte aligned");
  HIPCHK(c, sd::quantize_rows_e4m3(S(stream), static_cast<const bf16*>(w), (int)N, (int)K,
                                   static_cast<unsigned char*>(codes), scale));
  return SPECDEC_OK;
}

int specdec_get_row_stats(specdec_ctx* c, float* stats, void* stream) {
  int rc = check_ready(c, SPECDEC_VERIFIER, false);
  if (rc) return rc;
  if (!stats) return fail(c, SPECDEC_ERR_INVALID_ARG, "null stats");
  if (c->last_T <= 0) return fail(c, SPECDEC_ERR_BAD_STATE, "no verification pass to report");
  const size_t n = (size_t)c->B * c->last_T * SPECDEC_ROW_STATS;
  HIPCHK(c, hipMemcpyAsync(stats, c->last_row_stats, n * sizeof(float), hipMemcpyDeviceToDevice, S(stream)));
  return SPECDEC_OK;
}

}  // extern "C"
