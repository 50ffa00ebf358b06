#!/usr/bin/env python3
"""Benchmark of the SpecDec verification hot path on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W]

One *step* = one pass of the hot path over one batch: specdec_verify (row assembly, KV-cached
decoder pass with KV append, fused vocabulary projection + top-beta/tau acceptance) followed
by specdec_commit and a rewind to the starting lengths so that every step does the same work.
Workload: the batch-128 verification step of the translation-shaped loop (big verifier
6 layers, d=1024, 16 heads, FFN 4096, vocab 32768; B=128, k=10, 64 tokens already decoded,
source lengths uniform in [16,128], beta=3, tau=1.0).  Drafts are the verifier's own greedy
continuation (obtained with this library) with each slot replaced by a uniform-random token
with probability 0.2, which gives paper-shaped acceptance instead of the ~0 of untrained
random weights.  Inputs are seeded and synthetic and resident in HBM before timing starts.

Prints ONE JSON line; `value` = verified (committed) tokens per second.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

PEAK_HBM_GBS = 8000.0
PEAK_BF16_TFLOPS = 2500.0
SEED = 0


def _build_state(sd, synth, ses, desc, B, k, L, src_len, seed):
    """Decoded-so-far state of every sequence, built by the library itself: stream tokens are
    forced through verify+commit (accept_len and next_token given by the caller), so the KV
    cache holds the model's own keys/values for them."""
    import torch
    dev = ses.device
    S = int(src_len.max())
    sd.specdec_begin(ses.ctx, B, 10 ** 6)
    mem = ses.bf16(synth.make_memory(seed, B, S, desc.d_model))
    sd.specdec_set_memory(ses.ctx, sd.SPECDEC_VERIFIER, mem, ses.i32(src_len))
    prefix = synth.random_tokens(seed, "prefix", (B, L + 1), desc)     # u_1..u_L used
    acc = torch.zeros(B, dtype=torch.int32, device=dev)
    nxt = torch.zeros(B, dtype=torch.int32, device=dev)
    j = 0
    while j < L:
        a = min(k, L - j - 1)
        d = np.full((B, k), desc.pad_id, np.int32)
        d[:, :a] = prefix[:, j + 1:j + 1 + a]
        sd.specdec_verify(ses.ctx, ses.i32(d), k, 1, 0.0, acc, nxt)
        sd.specdec_commit(ses.ctx, ses.i32(np.full(B, a)), ses.i32(prefix[:, j + a + 1]))
        j += a + 1
    return mem


def _greedy_continuation(sd, synth, ses, desc, B, k, L, n, seed):
    """n greedy tokens per sequence from the current state (strict rule, accept nothing:
    every iteration commits the verifier's own next token), then rewind."""
    import torch
    dev = ses.device
    acc = torch.zeros(B, dtype=torch.int32, device=dev)
    nxt = torch.zeros(B, dtype=torch.int32, device=dev)
    zero = torch.zeros(B, dtype=torch.int32, device=dev)
    rnd = ses.i32(synth.random_tokens(seed, "scratch_drafts", (B, k), desc, full_vocab=True))
    for _ in range(n):
        sd.specdec_verify(ses.ctx, rnd, k, 1, 0.0, acc, nxt)
        sd.specdec_commit(ses.ctx, zero, nxt)
    toks = torch.zeros((B, L + n), dtype=torch.int32, device=dev)
    olen = torch.zeros(B, dtype=torch.int32, device=dev)
    sd.specdec_get_output(ses.ctx, toks, olen)
    torch.cuda.synchronize()
    sd.specdec_rewind(ses.ctx, ses.i32(np.full(B, L)))
    return toks[:, L:L + n].cpu().numpy()


def _timed(torch, fn, steps, warmup):
    for _ in range(warmup):
        fn()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(steps):
        fn()
    torch.cuda.synchronize()
    return (time.perf_counter() - t0) / steps


def kind_work(desc, R, B, k, L, src_len):
    """Algorithmic flops / bytes of ONE launch of each kernel kind (average over the launches
    of that kind in a step).  R = B*(k+1) real rows; padding and recomputation do not count."""
    d, F, V, H = desc.d_model, desc.d_ffn, desc.vocab, desc.n_heads
    T = k + 1
    self_keys = B * (L + T)                       # key rows streamed per layer (all heads)
    cross_keys = int(src_len.sum())
    kv_bytes = (self_keys + cross_keys) * d * 2 * 2 / 2.0   # K and V, bf16, per launch (2 launches/layer)
    return {
        "gemm_f32": ("mfma", (4 * R * d * d + 2 * R * d * F) / 3.0),
        "gemm_bf16": ("mfma", (2 * R * d * d + 2 * R * d * F) / 2.0),
        "gemm_qkv": ("mfma", 6.0 * R * d * d),
        "vocab": ("mfma", 2.0 * R * V * d),
        "attn": ("hbm", kv_bytes),
    }


def batch1_latency(sd, synth, torch, steps=200):
    """Single verify step at batch 1 (base verifier, memory 32, 16 tokens decoded, k=5)."""
    desc = synth.base_verifier(max_src=32, max_tgt=64, enc_layers=0)
    B, k, L = 1, 5, 16
    ses = sd.Session(B, k, 32, 64)
    w = ses.upload_weights(synth.make_weights(desc, SEED))
    ses.bind_model(sd.SPECDEC_VERIFIER, desc, w)
    _build_state(sd, synth, ses, desc, B, k, L, np.full(B, 32, np.int32), SEED)
    dr = ses.i32(synth.random_tokens(SEED, "drafts", (B, k), desc, full_vocab=True))
    acc = torch.zeros(B, dtype=torch.int32, device=ses.device)
    nxt = torch.zeros_like(acc)
    sec = _timed(torch, lambda: sd.specdec_verify(ses.ctx, dr, k, 3, 1.0, acc, nxt), steps, 20)
    d, F, V = desc.d_model, desc.d_ffn, desc.vocab
    wbytes = 2 * (desc.dec_layers * (3 * d * d + d * d + d * d + d * d + 2 * d * F) + V * d)
    kvbytes = 2 * 2 * desc.dec_layers * ((L + k + 1) + 32) * d
    ses.close()
    return {"workload": "single verify step: base verifier 6L d512, B=1, memory 32, 16 decoded, k=5",
            "verify_us": sec * 1e6, "algorithmic_bytes": wbytes + kvbytes,
            "hbm_frac": (wbytes + kvbytes) / sec / (PEAK_HBM_GBS * 1e9)}


def cpu_baseline(desc, B_sample, k, L, src_len, beta, tau, budget_s=20.0):
    """The CPU oracle, as it stands, on the first B_sample sequences of the same workload."""
    sys.path.insert(0, os.path.join(ROOT, "oracle"))
    import specdec_oracle as orc
    from paper_2203_16487_amd import synth
    try:
        from threadpoolctl import threadpool_info
        threads = max([p.get("num_threads", 1) for p in threadpool_info()] or [1])
    except Exception:
        threads = os.cpu_count() or 1
    model = orc.Model(desc, synth.weights_f32(synth.make_weights(desc, SEED)))
    S = int(src_len.max())
    mem = synth.make_memory(SEED, len(src_len), S, desc.d_model)
    prefix = synth.random_tokens(SEED, "prefix", (len(src_len), L + 1), desc)
    states, drafts = [], []
    for b in range(B_sample):
        st = orc.new_state(model, mem[b, :src_len[b]], L + 2 * k + 2)
        toks = [desc.bos_id] + list(prefix[b, 1:L + 1])
        n = len(toks) - 1
        orc.decoder_rows(model, st, toks[:-1], np.tril(np.ones((n, n), dtype=bool)))
        st.len += n
        g, t, s2 = [], toks[-1], st.clone()
        for _ in range(k):
            t = int(np.argmax(orc.dec_step(model, s2, t)))
            g.append(t)
        states.append((st, toks[-1]))
        drafts.append(g)
    drafts = synth.corrupt(SEED, "corrupt", np.array(drafts, np.int32), 0.2, desc)
    committed, reps, t0 = 0, 0, time.perf_counter()
    while True:
        for b in range(B_sample):
            st, pending = states[b]
            z = orc.verify_onepass(model, st, pending, list(drafts[b]))
            a, nx = orc.accept(z, list(drafts[b]), beta, tau)
            committed += a + 1            # commit = a + 1 tokens; rollback = len unchanged here
        reps += 1
        el = time.perf_counter() - t0
        if el >= budget_s / 2 or reps >= 400:
            break
    return {"value": committed / el, "unit": "tokens/s", "cores": int(threads), "kind": "oracle",
            "sample": f"first {B_sample} of the 128 sequences, verify+accept+commit repeated {reps}x "
                      f"({el:.1f} s of CPU work; setup untimed)"}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-batch1", action="store_true")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build runs on ONE GPU only (sequences are independent; more GPUs would "
              "each take a slice of the batch with no exchange). Use --gpus 1.", file=sys.stderr)
        sys.exit(2)

    import torch
    from paper_2203_16487_amd import binding as sd
    from paper_2203_16487_amd import synth
    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(1)
    sd.lib()   # fails loudly if the HIP library is missing

    B, k, L, beta, tau = 128, 10, 64, 3, 1.0
    desc = synth.big_verifier(max_src=128, max_tgt=128, enc_layers=0)
    src_len = synth.random_lengths(SEED, "src_len", B, 16, 128)
    ses = sd.Session(B, k, 128, 128)
    w = ses.upload_weights(synth.make_weights(desc, SEED))
    ses.bind_model(sd.SPECDEC_VERIFIER, desc, w)
    _build_state(sd, synth, ses, desc, B, k, L, src_len, SEED)
    greedy = _greedy_continuation(sd, synth, ses, desc, B, k, L, k, SEED)
    drafts = ses.i32(synth.corrupt(SEED, "corrupt", greedy, 0.2, desc))
    dev = ses.device
    acc = torch.zeros(B, dtype=torch.int32, device=dev)
    nxt = torch.zeros(B, dtype=torch.int32, device=dev)
    len0 = ses.i32(np.full(B, L))

    def step():
        sd.specdec_verify(ses.ctx, drafts, k, beta, tau, acc, nxt)
        sd.specdec_commit(ses.ctx, acc, nxt)
        sd.specdec_rewind(ses.ctx, len0)

    # rank the kernel kinds by time (one short pass per kind), then time the dominant one
    # with events inside a full timed region of its own
    work = kind_work(desc, B * (k + 1), B, k, L, src_len)
    per_kind = {}
    for name in work:
        sd.specdec_profile_select(ses.ctx, sd.KIND[name])
        for _ in range(3):
            step()
        ms, n = sd.specdec_profile_read(ses.ctx)
        per_kind[name] = (ms / 3.0, ms / max(n, 1))
    dominant = max(per_kind, key=lambda kname: per_kind[kname][0])
    sd.specdec_profile_select(ses.ctx, sd.KIND["none"])

    sec = _timed(torch, step, args.steps, args.warmup)
    tokens_per_step = int((acc + 1).sum().item())

    sd.specdec_profile_select(ses.ctx, sd.KIND[dominant])
    prof_steps = max(1, min(args.steps, 4000 // max(1, int(round(per_kind[dominant][0] / max(per_kind[dominant][1], 1e-9))))))
    _timed(torch, step, prof_steps, 2)
    ms, n = sd.specdec_profile_read(ses.ctx)
    sd.specdec_profile_select(ses.ctx, sd.KIND["none"])
    avg_s = ms / max(n, 1) * 1e-3
    bound, amount = work[dominant]
    if bound == "mfma":
        roof = {"bound": "mfma", "kernel": dominant, "achieved": amount / avg_s / 1e12, "peak": PEAK_BF16_TFLOPS,
                "unit": "TFLOP/s", "frac": amount / avg_s / 1e12 / PEAK_BF16_TFLOPS, "traffic": None,
                "avg_launch_us": avg_s * 1e6, "launches_timed": n}
    else:
        roof = {"bound": "hbm", "kernel": dominant, "achieved": amount / avg_s / 1e9, "peak": PEAK_HBM_GBS,
                "unit": "GB/s", "frac": amount / avg_s / 1e9 / PEAK_HBM_GBS, "traffic": None,
                "avg_launch_us": avg_s * 1e6, "launches_timed": n}

    d, F, V = desc.d_model, desc.d_ffn, desc.vocab
    R = B * (k + 1)
    step_flops = R * 2.0 * (desc.dec_layers * (3 * d * d + 3 * d * d + 2 * d * F) + V * d)
    out = {
        "metric": "verified tokens/sec (+ verify-step latency in us at batch 1 and 128)",
        "value": tokens_per_step / sec, "unit": "tokens/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": sec * 1e3, "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
        "config": {"workload": "translation-shaped loop, batch-128 verify+commit step: big verifier 6L d1024 H16 "
                               "F4096 V32768, B=128, k=10, 64 tokens decoded, source len U[16,128], beta=3 tau=1.0, "
                               "drafts = verifier greedy continuation with 20% random replacement",
                   "tokens_per_step": tokens_per_step, "seed": SEED},
        "batch128": {"verify_commit_us": sec * 1e6, "step_tflops": step_flops / sec / 1e12,
                     "mfma_frac": step_flops / sec / 1e12 / PEAK_BF16_TFLOPS,
                     "kernel_ms_per_step": {kname: round(v[0], 4) for kname, v in per_kind.items()}},
        "roofline": roof,
    }
    ses.close()
    if not args.no_batch1:
        out["batch1"] = batch1_latency(sd, synth, torch)
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(desc, 8, k, L, src_len, beta, tau)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
