"""Plain CPU oracle for SpecDec's draft-then-verify decoding (arXiv 2203.16487).

TEST INFRASTRUCTURE ONLY.  This file is the slow, obviously-correct definition
that the HIP library is checked against.  Only tests, the smoke check and the
benchmark's CPU-baseline leg may import it; the product path never does, and
this file imports nothing from the product.  It shares no code, tables or
helpers with the GPU implementation.

Everything works on ONE sequence at a time (batching = a Python loop, so batch
invariance holds by construction) and computes in the dtype of the weights it
is handed (fp32 in the parity tests; fp64 may be passed to size rounding error).

What follows the paper, and where:
  * verification = one parallel pass of the AR model over the k drafted tokens,
    equal by definition to k sequential AR steps              (Sec. 2, Eq. 2)
  * strict acceptance / bifurcation position c                 (Sec. 2, Eq. 1, 3)
  * relaxed top-beta / tau acceptance                          (Sec. 3.2, Eq. 8-10)
  * Spec-Drafter inference: prefix + k [MASK] slots, argmax    (Sec. 3.1.3, Eq. 7)
  * head-based drafting (the Blockwise Decoding comparison)    (Sec. 2 "Draft", Table 2)
  * loop: draft, verify, commit until EOS or the length cap    (Sec. 2)
  * Tok. = accepted tokens per iteration                       (Sec. 3.1.1, Eq. 4)

The paper names the architecture only as a 6+6 Transformer-base of 512/2048
(Sec. 4.1 "Model Configuration") run with fairseq.  The readings taken here:
post-LN sublayers, LayerNorm eps 1e-5 with biased variance, biases on every
linear map, interleaved sinusoidal positions starting at 0, embeddings scaled by
sqrt(d), one tied V x d matrix for input embedding and output projection,
attention scores scaled by 1/sqrt(d_head), ReLU, no final LayerNorm.

Pins (tests/test_oracle_*.py): one-pass == sequential; beta=1,tau=0 loop ==
greedy AR; acceptance vs brute-force sort on tiny vocabularies; layer math vs
torch.nn.TransformerDecoderLayer / TransformerEncoderLayer; the worked example
of the paper's case study (App. "Case Study", Table 14) as an accept pattern.
Unpinned: logits/Tok./BLEU of the trained models (no weights or data exist here).
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import Callable, Dict, List, Optional, Sequence, Tuple

import numpy as np

LN_EPS = 1e-5


# ----------------------------------------------------------------------------- model
@dataclass
class Model:
    """desc: any object with enc_layers, dec_layers, d_model, n_heads, d_ffn, vocab,
    bos_id, eos_id, pad_id, mask_id.  w: name -> ndarray, matrices [out, in]."""
    desc: object
    w: Dict[str, np.ndarray]

    @property
    def dtype(self):
        return self.w["embed"].dtype


def linear(x, w, b):
    return x @ w.T + b


def layer_norm(x, g, b):
    mu = x.mean(axis=-1, keepdims=True)
    var = ((x - mu) ** 2).mean(axis=-1, keepdims=True)        # biased variance
    return (x - mu) / np.sqrt(var + x.dtype.type(LN_EPS)) * g + b


def positional_encoding(positions, d, dtype):
    """PE(p, 2i) = sin(p / 10000^(2i/d)), PE(p, 2i+1) = cos(same)."""
    p = np.asarray(positions, dtype=np.float64)[:, None]
    i = np.arange(d // 2, dtype=np.float64)[None, :]
    ang = p / np.power(10000.0, 2.0 * i / d)
    pe = np.empty((p.shape[0], d), dtype=np.float64)
    pe[:, 0::2] = np.sin(ang)
    pe[:, 1::2] = np.cos(ang)
    return pe.astype(dtype)


def embed(model: Model, tokens, positions):
    d = model.desc.d_model
    e = model.w["embed"][np.asarray(tokens, dtype=np.int64)]
    return e * model.dtype.type(np.sqrt(d)) + positional_encoding(positions, d, model.dtype)


def attention(q, K, V, n_heads, visible):
    """Multi-head scaled dot-product attention.
    q [T,d]; K,V [n,d]; visible [T,n] bool (True = query row may look at key).
    Every row must see at least one key."""
    T, d = q.shape
    n = K.shape[0]
    dh = d // n_heads
    out = np.empty_like(q)
    scale = q.dtype.type(1.0 / np.sqrt(dh))
    for h in range(n_heads):
        sl = slice(h * dh, (h + 1) * dh)
        s = (q[:, sl] @ K[:, sl].T) * scale                   # [T,n]
        s = np.where(visible, s, -np.inf)
        s = s - s.max(axis=-1, keepdims=True)
        p = np.exp(s)
        p = p / p.sum(axis=-1, keepdims=True)
        out[:, sl] = p @ V[:, sl]
    return out


# ----------------------------------------------------------------------------- encoder
def encode(model: Model, src_tokens) -> np.ndarray:
    """Post-LN Transformer encoder over one unpadded source -> memory [S,d].
    (The encoder is run once per input: Sec. 3.1.2.)"""
    S = len(src_tokens)
    H = model.desc.n_heads
    d = model.desc.d_model
    w = model.w
    x = embed(model, src_tokens, np.arange(S))
    vis = np.ones((S, S), dtype=bool)
    for l in range(model.desc.enc_layers):
        p = f"enc.{l}"
        qkv = linear(x, w[p + ".attn.wqkv"], w[p + ".attn.bqkv"])
        a = attention(qkv[:, :d], qkv[:, d:2 * d], qkv[:, 2 * d:], H, vis)
        x = layer_norm(x + linear(a, w[p + ".attn.wo"], w[p + ".attn.bo"]),
                       w[p + ".ln1.g"], w[p + ".ln1.b"])
        hdn = np.maximum(linear(x, w[p + ".ffn.w1"], w[p + ".ffn.b1"]), 0)
        x = layer_norm(x + linear(hdn, w[p + ".ffn.w2"], w[p + ".ffn.b2"]),
                       w[p + ".ln2.g"], w[p + ".ln2.b"])
    return x


def cross_kv(model: Model, memory) -> Tuple[List[np.ndarray], List[np.ndarray]]:
    """Per decoder layer, keys and values of the encoder memory (computed once)."""
    d = model.desc.d_model
    Ks, Vs = [], []
    for l in range(model.desc.dec_layers):
        kv = linear(memory, model.w[f"dec.{l}.cross.wkv"], model.w[f"dec.{l}.cross.bkv"])
        Ks.append(kv[:, :d].copy())
        Vs.append(kv[:, d:].copy())
    return Ks, Vs


# ----------------------------------------------------------------------------- decoder state
@dataclass
class DecState:
    """Decoding state of one sequence for one model.
    K[l], V[l]: [cap, d] self-attention cache; rows [0, len) are valid, rows at and
    beyond len are dead (a verify pass writes rows there, commit decides how many
    become valid: that is the whole 'rollback')."""
    K: List[np.ndarray]
    V: List[np.ndarray]
    Kx: List[np.ndarray]
    Vx: List[np.ndarray]
    len: int = 0

    def clone(self) -> "DecState":
        return DecState([a.copy() for a in self.K], [a.copy() for a in self.V],
                        self.Kx, self.Vx, self.len)


def new_state(model: Model, memory, cap: int) -> DecState:
    d, L = model.desc.d_model, model.desc.dec_layers
    Kx, Vx = cross_kv(model, memory)
    z = lambda: np.zeros((cap, d), dtype=model.dtype)
    return DecState([z() for _ in range(L)], [z() for _ in range(L)], Kx, Vx, 0)


def decoder_rows(model: Model, st: DecState, tokens, block_visible) -> np.ndarray:
    """Run the decoder over T new rows placed at positions len..len+T-1.

    block_visible [T,T] bool: which of the T new rows each new row may attend to
    (all len cached rows are always visible).  Writes the new rows' K/V into the
    cache at len..len+T-1 WITHOUT advancing len.  Returns final hidden states [T,d].
    """
    w, dsc = model.w, model.desc
    d, H = dsc.d_model, dsc.n_heads
    T, n0 = len(tokens), st.len
    x = embed(model, tokens, np.arange(n0, n0 + T))
    vis_self = np.concatenate([np.ones((T, n0), dtype=bool), np.asarray(block_visible, bool)], axis=1)
    S = st.Kx[0].shape[0]
    vis_cross = np.ones((T, S), dtype=bool)
    for l in range(dsc.dec_layers):
        p = f"dec.{l}"
        qkv = linear(x, w[p + ".self.wqkv"], w[p + ".self.bqkv"])
        st.K[l][n0:n0 + T] = qkv[:, d:2 * d]
        st.V[l][n0:n0 + T] = qkv[:, 2 * d:]
        a = attention(qkv[:, :d], st.K[l][:n0 + T], st.V[l][:n0 + T], H, vis_self)
        x = layer_norm(x + linear(a, w[p + ".self.wo"], w[p + ".self.bo"]),
                       w[p + ".ln1.g"], w[p + ".ln1.b"])
        q = linear(x, w[p + ".cross.wq"], w[p + ".cross.bq"])
        a = attention(q, st.Kx[l], st.Vx[l], H, vis_cross)
        x = layer_norm(x + linear(a, w[p + ".cross.wo"], w[p + ".cross.bo"]),
                       w[p + ".ln2.g"], w[p + ".ln2.b"])
        hdn = np.maximum(linear(x, w[p + ".ffn.w1"], w[p + ".ffn.b1"]), 0)
        x = layer_norm(x + linear(hdn, w[p + ".ffn.w2"], w[p + ".ffn.b2"]),
                       w[p + ".ln3.g"], w[p + ".ln3.b"])
    return x


def vocab_logits(model: Model, h):
    return h @ model.w.get("embed_out", model.w["embed"]).T


def log_softmax(z):
    m = z.max(axis=-1, keepdims=True)
    return z - (m + np.log(np.exp(z - m).sum(axis=-1, keepdims=True)))


def dec_step(model: Model, st: DecState, token: int) -> np.ndarray:
    """One KV-cached autoregressive step: feed `token` at position len, return the
    logits of the next token [V] and advance len by one."""
    h = decoder_rows(model, st, [token], np.ones((1, 1), dtype=bool))
    st.len += 1
    return vocab_logits(model, h)[0]


# ----------------------------------------------------------------------------- verification
def verify_sequential(model: Model, st: DecState, pending: int, drafts) -> np.ndarray:
    """The definition (Eq. 2): k+1 sequential AR steps fed pending, y~_1..y~_k.
    Row i is the next-token distribution after pending and the first i drafts.
    Leaves st.len unchanged; cache rows len..len+k hold the fed tokens' K/V."""
    n0 = st.len
    rows = [dec_step(model, st, t) for t in [pending] + list(drafts)]
    st.len = n0
    return np.stack(rows)


def verify_onepass(model: Model, st: DecState, pending: int, drafts, return_hidden: bool = False):
    """The same k+1 rows of logits from ONE causal pass over [pending, drafts]
    (return_hidden: also the final hidden states [k+1, d] the logits were taken from)."""
    T = len(drafts) + 1
    h = decoder_rows(model, st, [pending] + list(drafts), np.tril(np.ones((T, T), dtype=bool)))
    return (vocab_logits(model, h), h) if return_hidden else vocab_logits(model, h)


def accept(logits, drafts, beta: int, tau: float) -> Tuple[int, int]:
    """Spec-Verification (Eq. 8-10).  Draft i (1-based) sits against row i-1.
    It is accepted iff all earlier drafts were, its log-probability is at least that
    of the beta-th ranked token (Eq. 8) and the top-1 log-probability exceeds it by
    at most tau (Eq. 9).  beta=1, tau=0 is the strict rule of Eq. 1-2.
    Returns (a, next): a = number of accepted drafts, next = the verifier's own
    token at the bifurcation row a (lowest index among maxima).  If every draft is
    accepted the row after the last draft supplies one more token."""
    logp = log_softmax(np.asarray(logits))
    a = 0
    for i, t in enumerate(drafts):
        s = np.sort(logp[i])[::-1]
        if logp[i, t] >= s[beta - 1] and s[0] - logp[i, t] <= logits.dtype.type(tau):
            a += 1
        else:
            break
    return a, int(np.argmax(logp[a]))


# ----------------------------------------------------------------------------- sequence bookkeeping
@dataclass
class SeqState:
    """stream = decoder input stream u_0..u_j: u_0 = BOS (or a given prefix), then the
    committed tokens.  The verifier has K/V for u_0..u_{j-1}; u_j is 'pending'."""
    stream: List[int]
    n_committed: int = 0          # tokens committed by decoding (excludes a given prefix)
    finished: bool = False


def commit(seq: SeqState, vst: DecState, drafts, a: int, nxt: int, eos_id: int, max_tgt: int) -> int:
    """Eq. 3: the iteration's output is the a accepted drafts followed by the
    verifier's token.  Stops after the first EOS or at max_tgt committed tokens;
    what follows is dropped.  The verifier cache keeps exactly the rows whose input
    tokens stay in the stream.  Returns the number of tokens appended."""
    n = 0
    for t in list(drafts[:a]) + [nxt]:
        seq.stream.append(int(t))
        seq.n_committed += 1
        n += 1
        if t == eos_id or seq.n_committed >= max_tgt:
            seq.finished = True
            break
    vst.len += n
    return n


# ----------------------------------------------------------------------------- drafter
def draft(model: Model, dst: DecState, stream: Sequence[int], k: int, return_logits: bool = False):
    """Spec-Drafter inference (Eq. 7): append k [MASK] tokens to the decoded stream
    and predict all of them in one pass.

    Prefix-LM reading of Eq. 7 (the slots are predicted from the decoded prefix and the source):
    committed rows attend causally among themselves (so their K/V never changes and
    is cached once); the k mask rows attend to every committed row and to all k mask
    rows.  Mask slot i sits at the position of the token it predicts.  Committed
    rows not yet cached (stream[dst.len:]) are processed in the same pass and their
    K/V kept; the mask rows' K/V is dropped."""
    new = list(stream[dst.len:])
    n = len(new)
    T = n + k
    vis = np.zeros((T, T), dtype=bool)
    vis[:n, :n] = np.tril(np.ones((n, n), dtype=bool))
    vis[n:, :] = True
    h = decoder_rows(model, dst, new + [model.desc.mask_id] * k, vis)
    dst.len += n
    z = vocab_logits(model, h[n:])
    toks = [int(t) for t in np.argmax(z, axis=-1)]
    return (toks, z) if return_logits else toks


def head_draft(model: Model, heads: Sequence[Dict[str, np.ndarray]], h: np.ndarray, return_logits: bool = False):
    """Head-based drafting (the drafter of Blockwise Decoding that Sec. 2 'Draft' and Table 2
    compare against): FFN heads on top of the target model's final hidden state h [d] of the
    last position, one per drafted token, all sharing the model's attention and its output
    embedding.  The paper gives no more than that; the reading taken: head i is a residual
    feed-forward block, h_i = h + W2_i relu(W1_i h + b1_i) + b2_i, its token is the arg-max of
    the tied output projection of h_i.  The model's own head (no block) predicts the next token;
    head i predicts the token i positions after it.
    heads: dicts with w1 [F,d], b1 [F], w2 [d,F], b2 [d].  Returns len(heads) tokens."""
    rows = [h + linear(np.maximum(linear(h, hd["w1"], hd["b1"]), 0), hd["w2"], hd["b2"]) for hd in heads]
    z = vocab_logits(model, np.stack(rows))
    toks = [int(t) for t in np.argmax(z, axis=-1)]
    return (toks, z) if return_logits else toks


# ----------------------------------------------------------------------------- reduced-precision weights
# Weight streaming in 8 bits (a precision / bandwidth variant of the verification pass, not part of
# the paper's method): a matrix is stored as OCP FP8 E4M3 codes (1 sign, 4 exponent bits with bias
# 7, 3 mantissa bits; no infinities; largest finite value 448) with one fp32 scale per output row,
# and multiplied as the up-cast values.  The oracle's side of it is the definition: what values
# the codes stand for, and which code a weight gets.
E4M3_MAX = 448.0


def e4m3_decode(codes: np.ndarray) -> np.ndarray:
    """Value of every E4M3 code: (-1)^s 2^(e-7) (1 + m/8) for e > 0, (-1)^s 2^-6 (m/8) for e = 0."""
    c = codes.astype(np.int64)
    s, e, m = (c >> 7) & 1, (c >> 3) & 15, c & 7
    mag = np.where(e > 0, np.ldexp(1.0 + m / 8.0, e - 7), np.ldexp(m / 8.0, -6))
    return np.where(s == 1, -mag, mag).astype(np.float32)


def e4m3_encode(x: np.ndarray) -> np.ndarray:
    """Nearest E4M3 code of fp32 values, ties to the even mantissa, magnitudes beyond 448 saturate
    to +-448 (code 0x7e / 0xfe: the all-ones mantissa at e = 15 is NaN and never produced)."""
    x = np.asarray(x, np.float32)
    sign = (np.signbit(x)).astype(np.uint8) << 7
    a = np.abs(x).astype(np.float32)
    bits = a.view(np.uint32).astype(np.int64)
    E = (bits >> 23) - 127
    mant = bits & 0x7FFFFF
    m = mant >> 20
    rem = mant & 0xFFFFF
    up = (rem > 0x80000) | ((rem == 0x80000) & ((m & 1) == 1))
    m = m + up
    carry = m == 8
    m = np.where(carry, 0, m)
    E = E + carry
    normal = ((E + 7) << 3) | m
    q = np.rint(a.astype(np.float64) * 512.0).astype(np.int64)       # subnormal grid: multiples of 2^-9 (rint: ties to even)
    sub = np.where(q >= 8, 0x08, q)
    code = np.where(a < np.float32(2.0 ** -6), sub, normal)
    code = np.where(a >= np.float32(E4M3_MAX), 0x7E, np.minimum(code, 0x7E))
    return (code.astype(np.uint8) | sign).astype(np.uint8)


def quantize_rows_e4m3(w: np.ndarray):
    """Per-output-row scaling: row n of w [N, K] is stored as codes of w[n] / s_n with
    s_n = max|w[n]| / 448 (1 for an all-zero row), all in fp32.  Returns (codes uint8 [N,K],
    scales fp32 [N], the values the codes stand for: decode(codes) * s_n, fp32 [N,K])."""
    w = np.asarray(w, np.float32)
    amax = np.abs(w).max(axis=1)
    s = np.where(amax > 0, amax / np.float32(E4M3_MAX), np.float32(1.0)).astype(np.float32)
    codes = e4m3_encode((w / s[:, None]).astype(np.float32))
    return codes, s, (e4m3_decode(codes) * s[:, None]).astype(np.float32)


def with_fp8_weights(model: Model) -> Model:
    """The model whose decoder projection matrices and (tied) output projection are the E4M3-stored
    values; biases, LayerNorm parameters, the cross K/V projection and the INPUT embedding rows
    stay as given.  Returns a model with an extra entry 'embed_out' used by vocab_logits."""
    w = dict(model.w)
    for name in list(w):
        if name.startswith("dec.") and name.split(".")[-1] in ("wqkv", "wo", "wq", "w1", "w2") and w[name].ndim == 2:
            w[name] = quantize_rows_e4m3(w[name])[2].astype(model.dtype)
    w["embed_out"] = quantize_rows_e4m3(w["embed"])[2].astype(model.dtype)
    return Model(model.desc, w)


def bf16_round(x: np.ndarray) -> np.ndarray:
    """fp32 values rounded to the nearest bf16 (8 significand bits, ties to even), returned as fp32."""
    u = np.ascontiguousarray(x, np.float32).view(np.uint32).astype(np.uint64)
    u = (u + 0x7FFF + ((u >> 16) & 1)) & 0xFFFF0000
    return u.astype(np.uint32).view(np.float32)


def with_fp8_cross_kv(model: Model, st: DecState) -> DecState:
    """The state whose cross-attention keys and values (computed once per input, read by every
    verification pass: the bulk of the bytes when the source is long) are the E4M3-stored values:
    each key's and each value's 64-wide per-head vector is one row of quantize_rows_e4m3 (its own
    fp32 scale).  Reading taken: the 8-bit store is a re-encoding of the 16-bit one, i.e. the codes
    are those of the keys / values as a bf16 tensor holds them (rounded to bf16 first), not of the
    unrounded projections.  The self-attention cache is untouched (shared, not copied)."""
    H, d = model.desc.n_heads, model.desc.d_model
    dh = d // H

    def q(a):
        S = a.shape[0]
        a16 = bf16_round(np.asarray(a, np.float32))
        return quantize_rows_e4m3(a16.reshape(S * H, dh))[2].reshape(S, d).astype(model.dtype)

    return DecState(st.K, st.V, [q(a) for a in st.Kx], [q(a) for a in st.Vx], st.len)


# ----------------------------------------------------------------------------- decoding loops
def greedy_decode(model: Model, memory, max_tgt: int, prefix: Optional[Sequence[int]] = None) -> List[int]:
    """Plain autoregressive greedy decoding from BOS (or a given input prefix)."""
    dsc = model.desc
    stream = list(prefix) if prefix is not None else [dsc.bos_id]
    st = new_state(model, memory, len(stream) + max_tgt + 1)
    for t in stream[:-1]:
        dec_step(model, st, t)
    out: List[int] = []
    tok = stream[-1]
    while len(out) < max_tgt:
        tok = int(np.argmax(dec_step(model, st, tok)))
        out.append(tok)
        if tok == dsc.eos_id:
            break
    return out


@dataclass
class LoopStats:
    iterations: int = 0
    committed: int = 0
    accepted: List[int] = field(default_factory=list)   # a per iteration

    @property
    def tok(self) -> float:                              # Eq. 4's Tok.
        return self.committed / max(1, self.iterations)


def specdec_decode(verifier: Model, memory_v, draft_fn: Callable[[List[int], int], List[int]],
                   k: int, beta: int, tau: float, max_tgt: int,
                   prefix: Optional[Sequence[int]] = None,
                   verify_fn: Optional[Callable] = None) -> Tuple[List[int], LoopStats]:
    """Draft-then-verify loop (Sec. 2): draft k tokens, verify them in one pass,
    keep the accepted drafts plus the verifier's token, repeat until EOS or max_tgt.
    draft_fn(stream, k) -> k token ids.  verify_fn defaults to verify_onepass."""
    dsc = verifier.desc
    stream = list(prefix) if prefix is not None else [dsc.bos_id]
    n_prefix = len(stream)
    vst = new_state(verifier, memory_v, n_prefix + max_tgt + k + 1)
    for t in stream[:-1]:
        dec_step(verifier, vst, t)
    seq = SeqState(stream)
    stats = LoopStats()
    vf = verify_fn or verify_onepass
    while not seq.finished:
        drafts = list(draft_fn(seq.stream, k))
        logits = vf(verifier, vst, seq.stream[-1], drafts)
        a, nxt = accept(logits, drafts, beta, tau)
        n = commit(seq, vst, drafts, a, nxt, dsc.eos_id, max_tgt)
        stats.iterations += 1
        stats.committed += n
        stats.accepted.append(a)
    return seq.stream[n_prefix:], stats


def make_drafter_fn(drafter: Model, memory_d, cap: int):
    """draft_fn backed by a Spec-Drafter model with its own cached state."""
    dst = new_state(drafter, memory_d, cap)
    return lambda stream, k: draft(drafter, dst, stream, k)
