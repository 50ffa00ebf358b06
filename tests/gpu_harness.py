"""Drives libspecdec through its C ABI for the parity tests (GPU only)."""
from __future__ import annotations

import numpy as np
import torch

from paper_2203_16487_amd import binding as sd
from paper_2203_16487_amd import synth
import cases


def open_verifier(case: cases.VerifyCase, k_max=None, max_tgt=None, max_batch=None, max_new=10 ** 6, options=None,
                  fill=0):
    """Session with the verifier bound, memory set, streams set and the oracle's cache loaded.
    options: {specdec_option: value} passed to specdec_configure; fill: byte the state and workspace
    buffers hold before they are bound."""
    k_max = k_max or case.k
    max_tgt = max_tgt or (case.L_max + case.k + 8)
    S = case.memory.shape[1]
    ses = sd.Session(max_batch or case.B, k_max, S, max_tgt, fill=fill)
    for opt, val in (options or {}).items():
        sd.specdec_configure(ses.ctx, opt, val)
    w = ses.upload_weights(case.bits)
    ses.bind_model(sd.SPECDEC_VERIFIER, case.desc, w)
    sd.specdec_begin(ses.ctx, case.B, max_new)
    sd.specdec_set_memory(ses.ctx, sd.SPECDEC_VERIFIER, ses.bf16(case.memory), ses.i32(case.src_len))
    sd.specdec_set_stream(ses.ctx, ses.i32(case.tokens), ses.i32(case.lens))
    L = max(case.L_max, 1)
    K, V = cases.oracle_flat_cache(case, L)
    sd.specdec_load_cache(ses.ctx, sd.SPECDEC_VERIFIER, ses.bf16(K), ses.bf16(V), ses.i32(case.lens))
    return ses


def gpu_verify(ses, case, drafts=None, want_logits=True, beta=None, tau=None):
    dev = ses.device
    B, k, V = case.B, case.k, case.desc.vocab
    d = ses.i32(case.drafts if drafts is None else drafts)
    acc = torch.full((B,), -7, dtype=torch.int32, device=dev)
    nxt = torch.full((B,), -7, dtype=torch.int32, device=dev)
    logits = torch.full((B, k + 1, V), float("nan"), dtype=torch.float32, device=dev) if want_logits else None
    sd.specdec_verify(ses.ctx, d, k, case.beta if beta is None else beta, case.tau if tau is None else tau,
                      acc, nxt, logits)
    stats = torch.zeros((B, k + 1, sd.ROW_STATS), dtype=torch.float32, device=dev)
    sd.specdec_get_row_stats(ses.ctx, stats)
    torch.cuda.synchronize()
    return dict(accept=acc.cpu().numpy(), next=nxt.cpu().numpy(),
                logits=None if logits is None else logits.cpu().numpy(), stats=stats.cpu().numpy(),
                accept_t=acc, next_t=nxt)


def gpu_cache(ses, case, L):
    Ld, d = case.desc.dec_layers, case.desc.d_model
    K = torch.zeros((Ld, case.B, L, d), dtype=torch.bfloat16, device=ses.device)
    V = torch.zeros_like(K)
    sd.specdec_get_cache(ses.ctx, sd.SPECDEC_VERIFIER, K, V)
    torch.cuda.synchronize()
    return K.float().cpu().numpy(), V.float().cpu().numpy()
