"""Builders of seeded verification cases: the oracle side (expected values) and the
marshalled arrays the GPU side consumes.  Test infrastructure only."""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import Dict, List, Optional

import numpy as np

from paper_2203_16487_amd import synth
import specdec_oracle as orc

NEAR = 1e-2          # near-threshold margin (log-likelihood units)


@dataclass
class VerifyCase:
    desc: synth.ModelDesc
    bits: Dict[str, np.ndarray]            # bf16 bit patterns, ABI order
    model: orc.Model
    B: int
    k: int
    beta: int
    tau: float
    memory: np.ndarray                     # [B,S,d] fp32 (bf16-representable)
    src_len: np.ndarray                    # [B]
    tokens: np.ndarray                     # [B, L_max+1] streams u_0..u_j (padded with pad)
    lens: np.ndarray                       # [B] j
    drafts: np.ndarray                     # [B,k]
    states: List[orc.DecState] = field(default_factory=list)   # oracle states, prefix cached
    # expected
    logits: Optional[np.ndarray] = None    # [B,k+1,V]
    accept: Optional[np.ndarray] = None
    nxt: Optional[np.ndarray] = None

    @property
    def L_max(self):
        return self.tokens.shape[1] - 1


def oracle_prefill(model: orc.Model, st: orc.DecState, tokens) -> None:
    """Cache K/V of `tokens` with one causal pass (== sequential steps, pinned in the oracle tests)."""
    n = len(tokens)
    if n:
        orc.decoder_rows(model, st, list(tokens), np.tril(np.ones((n, n), dtype=bool)))
        st.len += n


def make_verify_case(desc: synth.ModelDesc, seed: int, B: int, S: int, k: int, beta: int, tau: float,
                     len_lo: int, len_hi: int, drafts: str = "random", ragged_src: bool = False,
                     std: float = 0.02, corrupt_p: float = 0.2, cap_extra: int = 0, fp8: bool = False,
                     fp8_kv: bool = False) -> VerifyCase:
    """fp8: the expected values (prefix cache, greedy drafts, logits) come from the model whose decoder
    projection matrices and output matrix are stored as E4M3 codes with per-row scales; `bits` stay
    the bf16 weights the library is given.  fp8_kv: likewise with the cross-attention keys / values stored
    as E4M3 codes with one scale per (key, head) vector."""
    bits = synth.make_weights(desc, seed, std=std)
    model = orc.Model(desc, synth.weights_f32(bits))
    if fp8:
        model = orc.with_fp8_weights(model)
    memory = synth.make_memory(seed, B, S, desc.d_model)
    src_len = synth.random_lengths(seed, "src_len", B, 1, S) if ragged_src else np.full((B,), S, np.int32)
    lens = synth.random_lengths(seed, "prefix_len", B, len_lo, len_hi)
    L_max = int(lens.max())
    body = synth.random_tokens(seed, "prefix", (B, L_max + 1), desc)
    tokens = np.full((B, L_max + 1), desc.pad_id, np.int32)
    states = []
    for b in range(B):
        j = int(lens[b])
        tokens[b, :j + 1] = body[b, :j + 1]
        if j == 0:
            tokens[b, 0] = desc.bos_id
        st = orc.new_state(model, memory[b, :src_len[b]], j + k + 1 + cap_extra)
        if fp8_kv:
            st = orc.with_fp8_cross_kv(model, st)
        oracle_prefill(model, st, tokens[b, :j])
        states.append(st)
    if drafts == "random":
        dr = synth.random_tokens(seed, "drafts", (B, k), desc, full_vocab=True)
    else:
        # the verifier's own greedy continuation, each slot replaced by a random token w.p. corrupt_p
        dr = np.zeros((B, k), np.int32)
        for b in range(B):
            st = states[b].clone()
            t = int(tokens[b, lens[b]])
            for i in range(k):
                t = int(np.argmax(orc.dec_step(model, st, t)))
                dr[b, i] = t
        dr = synth.corrupt(seed, "corrupt", dr, corrupt_p, desc)
    return VerifyCase(desc, bits, model, B, k, beta, tau, memory, src_len, tokens, lens, dr, states)


def run_oracle(case: VerifyCase) -> None:
    V = case.desc.vocab
    case.logits = np.zeros((case.B, case.k + 1, V), np.float32)
    case.accept = np.zeros((case.B,), np.int32)
    case.nxt = np.zeros((case.B,), np.int32)
    for b in range(case.B):
        st = case.states[b]
        z = orc.verify_onepass(case.model, st, int(case.tokens[b, case.lens[b]]), list(case.drafts[b]))
        case.logits[b] = z
        a, n = orc.accept(z, list(case.drafts[b]), case.beta, case.tau)
        case.accept[b], case.nxt[b] = a, n


def oracle_flat_cache(case: VerifyCase, L: int):
    """Oracle K/V as [Ld, B, L, d] fp32 (rows beyond a state's capacity are zero)."""
    Ld, d = case.desc.dec_layers, case.desc.d_model
    K = np.zeros((Ld, case.B, L, d), np.float32)
    Vv = np.zeros_like(K)
    for b, st in enumerate(case.states):
        n = min(L, st.K[0].shape[0])
        for l in range(Ld):
            K[l, b, :n] = st.K[l][:n]
            Vv[l, b, :n] = st.V[l][:n]
    return K, Vv


def near_threshold_rows(z: np.ndarray, drafts, beta: int, tau: float):
    """Per row of one sequence's oracle logits: is the accept decision (rows < k) or the
    arg-max (all rows) within NEAR of flipping?"""
    k = len(drafts)
    near_acc = np.zeros(k, bool)
    near_arg = np.zeros(k + 1, bool)
    for i in range(k + 1):
        s = np.sort(z[i])[::-1]
        near_arg[i] = (s[0] - s[1]) <= NEAR
        if i < k:
            zd = z[i, drafts[i]]
            near_acc[i] = abs(zd - s[beta - 1]) <= NEAR or abs(tau - (s[0] - zd)) <= NEAR
            # a draft that is itself the beta-th ranked token sits exactly on the threshold by
            # construction; what can flip is its order with the next-ranked score
            if zd == s[beta - 1] and beta < len(s):
                near_acc[i] = (zd - s[beta]) <= NEAR or abs(tau - (s[0] - zd)) <= NEAR
    return near_acc, near_arg


def compare_decisions(case: VerifyCase, accept_gpu, next_gpu):
    """Returns (n_exact, n_excused, unexcused list).  A mismatch is excused only if the first
    row where the two sides part is near-threshold on the ORACLE's logits."""
    exact, excused, bad = 0, 0, []
    for b in range(case.B):
        a_o, n_o = int(case.accept[b]), int(case.nxt[b])
        a_g, n_g = int(accept_gpu[b]), int(next_gpu[b])
        if (a_o, n_o) == (a_g, n_g):
            exact += 1
            continue
        near_acc, near_arg = near_threshold_rows(case.logits[b], list(case.drafts[b]), case.beta, case.tau)
        if a_o != a_g:
            row = min(a_o, a_g)
            ok = row < case.k and near_acc[row]
        else:
            ok = near_arg[a_o]
        if ok:
            excused += 1
        else:
            bad.append((b, (a_o, n_o), (a_g, n_g)))
    return exact, excused, bad
