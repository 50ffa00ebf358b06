"""Further parity cases through the C ABI: the Spec-Drafter pass compared numerically (slot logits,
row statistics, appended keys/values), caches loaded short of the stream, non-finite garbage in
dead cache rows and in the caller's buffers, the prefix / counter / option entry points, and how
the logit error scales with the logit magnitude.

Tolerances: logits max-abs <= 2e-2 where the workload definition's shapes and weight scale apply
(d = 512 / 1024, std 0.02: logit std 0.45 / 0.64); in general the error is a fraction of the
logit scale (bf16 rounding of every GEMM input is relative), so a case with larger logits is held
to max-abs <= 4 % of the ORACLE's logit standard deviation instead.  Keys / values: 3e-2 (bf16
storage of values of magnitude ~3)."""
import numpy as np
import pytest
import torch

import cases
import gpu_harness as gh
import specdec_oracle as orc
import test_gpu_draft_loop as dl
from paper_2203_16487_amd import binding as sd
from paper_2203_16487_amd import synth

pytestmark = pytest.mark.gpu
LOGIT_TOL = 2e-2
KV_TOL = 3e-2
REL_TOL = 0.04          # of the oracle's logit standard deviation


def drafter_pass_case(dd, db, dm, B, S_max, k, lens, seed, prefill, sample=None, max_tgt=64, fixed_src=False,
                      options=None):
    """One Spec-Drafter pass of the whole batch on the GPU; the oracle recomputes `sample` (all
    by default).  Returns the worst logit / key-value errors seen."""
    src_len = np.full(B, S_max, np.int32) if fixed_src else synth.random_lengths(seed, "src_len", B, 2, S_max)
    src = synth.random_tokens(seed, "src", (B, S_max), dd)
    L_max = int(lens.max())
    toks = synth.random_tokens(seed, "stream", (B, L_max + 1), dd)
    toks[:, 0] = dd.bos_id
    ses = dl.open_session(B, k, S_max, max_tgt, dr=(dd, db), options=options)
    dev = ses.device
    sd.specdec_begin(ses.ctx, B, 100)
    sd.specdec_encode(ses.ctx, ses.i32(src), ses.i32(src_len))
    sd.specdec_set_stream(ses.ctx, ses.i32(toks), ses.i32(lens))
    if prefill:
        sd.specdec_prefill(ses.ctx, sd.SPECDEC_DRAFTER)
    dr = torch.full((B, k), -1, dtype=torch.int32, device=dev)
    logits = torch.full((B, k, dd.vocab), float("nan"), dtype=torch.float32, device=dev)
    sd.specdec_draft(ses.ctx, k, dr, logits)
    stats = torch.zeros((B, k, sd.ROW_STATS), dtype=torch.float32, device=dev)
    sd.specdec_get_draft_stats(ses.ctx, stats)
    L = L_max + 1
    Kg = torch.zeros((dd.dec_layers, B, L, dd.d_model), dtype=torch.bfloat16, device=dev)
    Vg = torch.zeros_like(Kg)
    sd.specdec_get_cache(ses.ctx, sd.SPECDEC_DRAFTER, Kg, Vg)
    # the pass without the parity pointer (arg-max only kernel) must give the same drafts
    dr2 = torch.full((B, k), -1, dtype=torch.int32, device=dev)
    sd.specdec_rewind(ses.ctx, ses.i32(lens))          # nothing committed: lengths unchanged, cached cut to j+1
    sd.specdec_draft(ses.ctx, k, dr2)
    torch.cuda.synchronize()
    g_dr, g_z, g_st = dr.cpu().numpy(), logits.cpu().numpy(), stats.cpu().numpy()
    assert np.array_equal(g_dr, dr2.cpu().numpy())
    Kg, Vg = Kg.float().cpu().numpy(), Vg.float().cpu().numpy()
    assert np.isfinite(g_z).all()
    # statistics are those of the library's own logits
    assert np.array_equal(g_st[..., 1].astype(np.int64), g_z.argmax(-1))
    assert np.array_equal(g_st[..., 0], g_z.max(-1))
    assert np.array_equal(g_dr, g_z.argmax(-1).astype(np.int32))
    worst_z, worst_kv, excused = 0.0, 0.0, 0
    for b in (range(B) if sample is None else sample):
        mem = orc.encode(dm, list(src[b, :src_len[b]]))
        dst = orc.new_state(dm, mem, max_tgt + k + 2)
        stream = [int(t) for t in toks[b, :lens[b] + 1]]
        t_o, z_o = orc.draft(dm, dst, stream, k, return_logits=True)
        err = float(np.abs(g_z[b] - z_o).max())
        worst_z = max(worst_z, err)
        assert err <= LOGIT_TOL, (b, err)
        excused += dl.check_drafts(g_dr[b:b + 1], [t_o], [z_o], f"drafter {b}")
        n = len(stream)                                    # stream rows now cached by the drafter
        for l in range(dd.dec_layers):
            e = max(float(np.abs(Kg[l, b, :n] - dst.K[l][:n]).max()), float(np.abs(Vg[l, b, :n] - dst.V[l][:n]).max()))
            worst_kv = max(worst_kv, e)
            assert e <= KV_TOL, (b, l, e)
    ses.close()
    return worst_z, worst_kv, excused


def test_drafter_pass_numerics_small():
    """Toy drafter (d = 128, std 0.08 weights): uncached streams of different lengths, ingested by the
    pass itself or by the prefill it triggers; slot logits, statistics and appended K/V vs the oracle."""
    _, (dd, db, dm) = dl.make_models(seed=12)
    lens = synth.random_lengths(12, "len", 6, 0, 20)
    wz, wkv, ex = drafter_pass_case(dd, db, dm, B=6, S_max=13, k=5, lens=lens, seed=12, prefill=False, max_tgt=48)
    print(f"[drafter numerics small] logits max-abs err {wz:.3e}, K/V {wkv:.3e}, {ex} near-ties excused")


def test_drafter_pass_numerics_config3_shape():
    """Spec-Drafter shape (12 + 2 layers, d = 512, V = 32768, source 128, 32 decoded, k = 10), B = 6."""
    dd = synth.spec_drafter(max_src=128, max_tgt=64)
    db = synth.make_weights(dd, 0, tag="drafter")
    dm = orc.Model(dd, synth.weights_f32(db))
    wz, wkv, ex = drafter_pass_case(dd, db, dm, B=6, S_max=128, k=10, lens=np.full(6, 32, np.int32), seed=0,
                                    prefill=True, fixed_src=True)
    print(f"[drafter numerics config3] logits max-abs err {wz:.3e}, K/V {wkv:.3e}, {ex} near-ties excused")


def test_drafter_pass_numerics_config3_full_batch():
    """The same at the full batch of 64 (the launch configuration of the benchmark's drafter pass),
    three sequences recomputed by the oracle."""
    dd = synth.spec_drafter(max_src=128, max_tgt=64)
    db = synth.make_weights(dd, 0, tag="drafter")
    dm = orc.Model(dd, synth.weights_f32(db))
    wz, wkv, ex = drafter_pass_case(dd, db, dm, B=64, S_max=128, k=10, lens=np.full(64, 32, np.int32), seed=0,
                                    prefill=True, sample=(0, 31, 63), fixed_src=True)
    print(f"[drafter numerics config3 B=64] logits max-abs err {wz:.3e}, K/V {wkv:.3e}, {ex} near-ties excused")


def small_case(seed, B=5, k=4, **kw):
    desc = synth.ModelDesc(0, 2, 128, 2, 256, 1000, 16, 64).resolved()
    args = dict(S=9, beta=3, tau=1.0, len_lo=3, len_hi=14, drafts="greedy", ragged_src=True, std=0.08)
    args.update(kw)
    return cases.make_verify_case(desc, seed=seed, B=B, k=k, **args)


def test_cache_loaded_short_of_the_stream_is_caught_on_device():
    """specdec_load_cache with n < j for some sequences: those report accept_len -1 / pad until a
    prefill has cached the missing rows; the others are unaffected.  Afterwards all match the oracle."""
    for B, k in ((5, 4), (40, 4)):                      # small-batch kernels / general kernels
        case = small_case(seed=51, B=B, k=k)
        cases.run_oracle(case)
        ses = gh.open_verifier(case)
        short = np.zeros(B, bool)
        short[[1, B - 1]] = True
        n = case.lens.copy()
        n[short] -= 2
        L = max(case.L_max, 1)
        K, V = cases.oracle_flat_cache(case, L)
        sd.specdec_set_stream(ses.ctx, ses.i32(case.tokens), ses.i32(case.lens))
        sd.specdec_load_cache(ses.ctx, sd.SPECDEC_VERIFIER, ses.bf16(K), ses.bf16(V), ses.i32(n))
        out = gh.gpu_verify(ses, case, want_logits=False)
        assert (out["accept"][short] == -1).all() and (out["next"][short] == case.desc.pad_id).all()
        assert np.array_equal(out["accept"][~short], case.accept[~short]) or not cases.compare_decisions(
            case, np.where(short, case.accept, out["accept"]), np.where(short, case.nxt, out["next"]))[2]
        # a commit of the refused sequences changes nothing
        sd.specdec_commit(ses.ctx, out["accept_t"], out["next_t"])
        sd.specdec_rewind(ses.ctx, ses.i32(case.lens))
        sd.specdec_prefill(ses.ctx, sd.SPECDEC_VERIFIER)
        out = gh.gpu_verify(ses, case)
        assert np.abs(out["logits"] - case.logits).max() <= LOGIT_TOL
        assert not cases.compare_decisions(case, out["accept"], out["next"])[2]
        ses.close()


def test_drafter_with_a_short_loaded_cache_returns_pad_drafts():
    """A drafter cache loaded more than one token short of the stream: the pass (sized for one new
    stream row per sequence) has no room for that sequence's mask slots, which must come back as
    pad_id, never as another sequence's rows."""
    _, (dd, db, dm) = dl.make_models(seed=13)
    B, S_max, k = 4, 9, 5
    lens = np.array([6, 9, 7, 8], np.int32)
    src_len = np.full(B, S_max, np.int32)
    src = synth.random_tokens(13, "src", (B, S_max), dd)
    toks = synth.random_tokens(13, "stream", (B, int(lens.max()) + 1), dd)
    toks[:, 0] = dd.bos_id
    ses = dl.open_session(B, k, S_max, 48, dr=(dd, db))
    dev = ses.device
    sd.specdec_begin(ses.ctx, B, 100)
    sd.specdec_encode(ses.ctx, ses.i32(src), ses.i32(src_len))
    sd.specdec_set_stream(ses.ctx, ses.i32(toks), ses.i32(lens))
    sd.specdec_prefill(ses.ctx, sd.SPECDEC_DRAFTER)
    L = int(lens.max()) + 1
    Kg = torch.zeros((dd.dec_layers, B, L, dd.d_model), dtype=torch.bfloat16, device=dev)
    Vg = torch.zeros_like(Kg)
    sd.specdec_get_cache(ses.ctx, sd.SPECDEC_DRAFTER, Kg, Vg)
    dr_full = torch.full((B, k), -1, dtype=torch.int32, device=dev)
    sd.specdec_draft(ses.ctx, k, dr_full)
    # same streams, cache of sequence 2 loaded three tokens short (n = j - 2 < j)
    n = lens.copy()
    n[2] -= 2
    sd.specdec_set_stream(ses.ctx, ses.i32(toks), ses.i32(lens))
    sd.specdec_load_cache(ses.ctx, sd.SPECDEC_DRAFTER, Kg, Vg, ses.i32(n))
    dr = torch.full((B, k), -1, dtype=torch.int32, device=dev)
    sd.specdec_draft(ses.ctx, k, dr)
    torch.cuda.synchronize()
    g, full = dr.cpu().numpy(), dr_full.cpu().numpy()
    assert (g[2] == dd.pad_id).all()
    assert np.array_equal(g[[0, 1, 3]], full[[0, 1, 3]])
    ses.close()


def test_dead_cache_rows_and_caller_buffers_may_hold_anything():
    """Rows at and beyond the cached length are dead (Sec. 2: drafts after the bifurcation are
    discarded): a cache loaded with NaN in every row >= n, into state and workspace buffers whose
    every untouched byte is 0xFF (NaN as bf16 and as fp32), gives finite logits equal to the clean
    run's to the last bit, on both kernel paths."""
    for B, k in ((3, 4), (40, 4)):
        case = small_case(seed=52, B=B, k=k, cap_extra=8)
        cases.run_oracle(case)
        ses0 = gh.open_verifier(case)
        clean = gh.gpu_verify(ses0, case)
        ses0.close()
        ses = gh.open_verifier(case, fill=0xFF)
        L = case.L_max + case.k + 6
        K, V = cases.oracle_flat_cache(case, L)
        for b in range(B):
            K[:, b, case.lens[b]:] = np.nan
            V[:, b, case.lens[b]:] = np.nan
        sd.specdec_load_cache(ses.ctx, sd.SPECDEC_VERIFIER, ses.bf16(K), ses.bf16(V), ses.i32(case.lens))
        out = gh.gpu_verify(ses, case)
        assert np.isfinite(out["logits"]).all()
        assert np.array_equal(out["logits"], clean["logits"])
        assert np.array_equal(out["accept"], clean["accept"]) and np.array_equal(out["next"], clean["next"])
        assert np.abs(out["logits"] - case.logits).max() <= LOGIT_TOL
        # rollback: commit, then verify again -- the rejected rows of the first pass (now beyond j)
        # and the NaN rows behind them must not reach the second pass
        sd.specdec_commit(ses.ctx, out["accept_t"], out["next_t"])
        out2 = gh.gpu_verify(ses, case, want_logits=True)
        assert np.isfinite(out2["logits"]).all()
        ses.close()


def test_set_prefix_counters_and_commit_clamp():
    """specdec_set_prefix = set_stream + load_cache in one call; the device counters follow the
    commits (Sec. 3.1.1 Eq. 4: tokens appended = sum over iterations of accepted + 1, minus
    truncation); an accept_len beyond the k of the latest pass is clamped to it."""
    case = small_case(seed=53, B=6, k=4, cap_extra=24)
    cases.run_oracle(case)
    k_max = 8
    S = case.memory.shape[1]
    ses = sd.Session(case.B, k_max, S, case.L_max + 40)
    ses.bind_model(sd.SPECDEC_VERIFIER, case.desc, ses.upload_weights(case.bits))
    sd.specdec_begin(ses.ctx, case.B, 10 ** 9)             # a cap far beyond the arena is clamped, not wrapped
    sd.specdec_set_memory(ses.ctx, sd.SPECDEC_VERIFIER, ses.bf16(case.memory), ses.i32(case.src_len))
    L = max(case.L_max, 1)
    K, V = cases.oracle_flat_cache(case, L)
    sd.specdec_set_prefix(ses.ctx, sd.SPECDEC_VERIFIER, ses.i32(case.tokens), ses.i32(case.lens), ses.bf16(K), ses.bf16(V))
    out = gh.gpu_verify(ses, case)
    assert np.abs(out["logits"] - case.logits).max() <= LOGIT_TOL
    assert not cases.compare_decisions(case, out["accept"], out["next"])[2]
    dev = ses.device
    fin = torch.zeros(case.B, dtype=torch.int32, device=dev)
    olen = torch.zeros(case.B, dtype=torch.int32, device=dev)
    toks = torch.zeros((case.B, 64), dtype=torch.int32, device=dev)
    # first a pass with k = 8 (fills all 8 stored drafts), then one with k = 4 committed with accept_len 8:
    # only 4 drafts + the next token may be appended
    d8 = synth.random_tokens(53, "d8", (case.B, 8), case.desc, full_vocab=True)
    acc = torch.zeros(case.B, dtype=torch.int32, device=dev)
    nxt = torch.zeros(case.B, dtype=torch.int32, device=dev)
    sd.specdec_verify(ses.ctx, ses.i32(d8), 8, 1, 0.0, acc, nxt)
    sd.specdec_verify(ses.ctx, ses.i32(case.drafts), 4, 1, 0.0, acc, nxt)
    sd.specdec_commit(ses.ctx, ses.i32(np.full(case.B, 8)), nxt)
    sd.specdec_get_output(ses.ctx, toks, olen, fin)
    cnt = torch.zeros(sd.SPECDEC_COUNTERS, dtype=torch.int32, device=dev)
    sd.specdec_get_counters(ses.ctx, cnt)
    torch.cuda.synchronize()
    eos = case.desc.eos_id
    want_total = 0
    for b in range(case.B):
        want = [int(t) for t in case.drafts[b]] + [int(nxt[b])]
        if eos in want:
            want = want[:want.index(eos) + 1]
        assert int(olen[b]) == len(want) and toks[b, :len(want)].cpu().tolist() == want, b
        want_total += len(want)
    c = cnt.cpu().numpy()
    assert c[0] == 1 and c[1] == want_total and c[2] == int(fin.sum())
    ses.close()


def test_logit_error_scales_with_logit_magnitude():
    """Transformer-base verifier shape (d = 512, F = 2048, 6 layers, V = 32768).  With the workload's
    weight scale (std 0.02) the absolute tolerance holds with margin; with std 0.05 the logits are
    2.5x larger and so is the error: it is held to 4 % of the oracle's logit standard deviation (bf16
    rounding of the GEMM inputs is a relative error), decisions stay exact up to the near-threshold rule."""
    desc = synth.base_verifier(max_src=32, max_tgt=64, enc_layers=0)
    for std, B, k, seed in ((0.02, 3, 9, 61), (0.02, 12, 2, 62), (0.05, 3, 9, 61), (0.05, 12, 2, 62)):
        case = cases.make_verify_case(desc, seed=seed, B=B, S=24, k=k, beta=3, tau=1.0, len_lo=2, len_hi=20,
                                      drafts="greedy", ragged_src=True, std=std)
        cases.run_oracle(case)
        ses = gh.open_verifier(case)
        out = gh.gpu_verify(ses, case)
        ses.close()
        err = float(np.abs(out["logits"] - case.logits).max())
        zstd = float(case.logits.std())
        print(f"[logit scale] std {std} B={B} k={k}: logit std {zstd:.3f}, max-abs err {err:.3e} = {err / zstd:.2%} of it")
        assert err <= REL_TOL * zstd
        if std == 0.02:
            assert err <= LOGIT_TOL
        assert not cases.compare_decisions(case, out["accept"], out["next"])[2]


def stacked_heads(ses, heads_bits):
    """per-head bf16 bit patterns -> the stacked device tensors specdec_bind_draft_heads takes"""
    def dev(a):
        return torch.from_numpy(np.ascontiguousarray(a).view(np.int16)).to(ses.device).view(torch.bfloat16)
    return (dev(np.concatenate([h["w1"] for h in heads_bits], 0)), dev(np.concatenate([h["b1"] for h in heads_bits], 0)),
            dev(np.stack([h["w2"] for h in heads_bits], 0)), dev(np.concatenate([h["b2"] for h in heads_bits], 0)))


def test_head_based_drafter_matches_oracle():
    """Head-based drafting (Sec. 2 'Draft', Table 2 first row) on top of the verifier: after a
    verification pass the heads' logits and tokens equal the oracle's, computed from the oracle's own
    hidden state at the row the library branched at; both kernel paths (25 and 200 rows)."""
    for B, k, nh, seed in ((5, 4, 4, 81), (40, 4, 3, 82)):
        case = small_case(seed=seed, B=B, k=k)
        hb = synth.make_head_weights(case.desc, nh, seed, std=0.08)
        heads = [synth.weights_f32(h) for h in hb]
        ses = gh.open_verifier(case)
        w = stacked_heads(ses, hb)
        sd.specdec_bind_draft_heads(ses.ctx, nh, *w)
        out = gh.gpu_verify(ses, case, want_logits=False)
        dr = torch.full((B, nh), -1, dtype=torch.int32, device=ses.device)
        zl = torch.full((B, nh, case.desc.vocab), float("nan"), dtype=torch.float32, device=ses.device)
        sd.specdec_draft_heads(ses.ctx, out["accept_t"], nh, dr, zl)
        torch.cuda.synchronize()
        g_dr, g_z = dr.cpu().numpy(), zl.cpu().numpy()
        worst, excused = 0.0, 0
        for b in range(B):
            z, h = orc.verify_onepass(case.model, case.states[b], int(case.tokens[b, case.lens[b]]), list(case.drafts[b]),
                                      return_hidden=True)
            a = int(out["accept"][b])
            t_o, z_o = orc.head_draft(case.model, heads, h[a], return_logits=True)
            err = float(np.abs(g_z[b] - z_o).max())
            worst = max(worst, err)
            # the heads have no LayerNorm after their residual sum: their logits are larger than the
            # verifier's (std ~1.3 here), so the bound is the relative one of this module's docstring
            assert err <= max(LOGIT_TOL, REL_TOL * float(z_o.std())), (b, err, float(z_o.std()))
            excused += dl.check_drafts(g_dr[b:b + 1], [t_o], [z_o], f"heads {b}")
        print(f"[head drafter B={B}] logits max-abs err {worst:.3e}, {excused} near-ties excused")
        ses.close()


def test_head_drafter_loop_strict_rule_reproduces_greedy():
    """Draft-then-verify with the heads as the drafter under the strict rule (beta = 1, tau = 0):
    whatever the heads propose, the committed tokens are the verifier's greedy decoding (Sec. 3.2)."""
    case = small_case(seed=83, B=4, k=3, cap_extra=40, len_lo=2, len_hi=6)
    hb = synth.make_head_weights(case.desc, 3, 83, std=0.08)
    ses = gh.open_verifier(case, max_tgt=case.L_max + 40, max_new=12)
    sd.specdec_bind_draft_heads(ses.ctx, 3, *stacked_heads(ses, hb))
    dev = ses.device
    B, k = case.B, 3
    acc = torch.zeros(B, dtype=torch.int32, device=dev)
    nxt = torch.zeros(B, dtype=torch.int32, device=dev)
    nact = torch.ones(1, dtype=torch.int32, device=dev)
    dr = ses.i32(case.drafts)
    for _ in range(14):
        sd.specdec_verify(ses.ctx, dr, k, 1, 0.0, acc, nxt)
        sd.specdec_draft_heads(ses.ctx, acc, k, dr)
        sd.specdec_commit(ses.ctx, acc, nxt, nact)
        if int(nact.item()) == 0:
            break
    toks = torch.zeros((B, 12), dtype=torch.int32, device=dev)
    olen = torch.zeros(B, dtype=torch.int32, device=dev)
    sd.specdec_get_output(ses.ctx, toks, olen)
    torch.cuda.synchronize()
    near = 0
    for b in range(B):
        prefix = [int(t) for t in case.tokens[b, :case.lens[b] + 1]]
        ref = orc.greedy_decode(case.model, case.memory[b, :case.src_len[b]], 12, prefix=prefix)
        got = toks[b, :int(olen[b])].cpu().tolist()
        if got != ref:
            # a near-tie in the verifier's own arg-max may fork the two decodings: check the fork is one
            i = next(j for j in range(min(len(got), len(ref))) if got[j] != ref[j])
            st = orc.new_state(case.model, case.memory[b, :case.src_len[b]], len(prefix) + 14)
            for t in (prefix + ref[:i])[:-1]:
                orc.dec_step(case.model, st, t)
            assert dl.near_tie(orc.dec_step(case.model, st, (prefix + ref[:i])[-1])), (b, i, got, ref)
            near += 1
    print(f"[head drafter loop] greedy output reproduced ({near} near-tie forks)")
    ses.close()


def test_large_drafter_shape_24_plus_6():
    """The drafter shape of the paper's large-model comparison (App. 'Comparison with Other Work': 24-layer
    encoder, 6-layer decoder, 1024 / 4096 / 16 heads), reduced batch and source for the CPU oracle."""
    dd = synth.ModelDesc(24, 6, 1024, 16, 4096, 32768, 48, 64).resolved()
    db = synth.make_weights(dd, 0, tag="drafter24")
    dm = orc.Model(dd, synth.weights_f32(db))
    wz, wkv, ex = drafter_pass_case(dd, db, dm, B=3, S_max=40, k=10, lens=np.array([7, 12, 3], np.int32), seed=5,
                                    prefill=False)
    print(f"[drafter 24+6] logits max-abs err {wz:.3e}, K/V {wkv:.3e}, {ex} near-ties excused")


def test_random_small_shapes_against_oracle_and_across_paths():
    """Sixteen seeded random small cases (batch 1-8, block size 1-15, prefixes 0-40, ragged sources, a
    pass of at most 32 rows): the fused small-batch kernels and the general kernels both against the
    oracle, and against each other (same tolerance: different kernels, same arithmetic up to
    rounding order)."""
    desc = synth.ModelDesc(0, 2, 128, 2, 256, 1000, 24, 64).resolved()
    rng = np.random.default_rng(2024)
    worst = 0.0
    for case_no in range(16):
        B = int(rng.integers(1, 9))
        k = int(rng.integers(1, min(15, 32 // B - 1) + 1))
        hi = int(rng.integers(0, 41))
        S = int(rng.integers(1, 25))
        case = small_case(seed=500 + case_no, B=B, k=k, S=S, len_lo=0, len_hi=hi, beta=int(rng.integers(1, 6)),
                          tau=float(rng.choice([0.0, 0.5, 1.0, 3.0])))
        cases.run_oracle(case)
        tol = max(LOGIT_TOL, REL_TOL * float(case.logits.std()))
        outs = {}
        for name, opt in (("fused", None), ("general", {sd.SPECDEC_OPT_SMALL_BATCH_KERNELS: 0})):
            ses = gh.open_verifier(case, options=opt)
            outs[name] = gh.gpu_verify(ses, case)
            ses.close()
            err = float(np.abs(outs[name]["logits"] - case.logits).max())
            worst = max(worst, err)
            assert err <= tol, (case_no, name, B, k, hi, S, err)
            assert not cases.compare_decisions(case, outs[name]["accept"], outs[name]["next"])[2], (case_no, name, B, k)
        assert np.abs(outs["fused"]["logits"] - outs["general"]["logits"]).max() <= tol, (case_no, B, k)
    print(f"[random shapes] 16 cases x 2 paths, worst max-abs logit err {worst:.3e}")


def test_wide_vocabulary_tiles_on_small_shapes():
    """The 256 x 256 vocabulary tiles (by default taken in the batched passes only) forced on shapes the
    oracle covers in full: rows that end inside a row tile or span two of them, vocabularies that end
    inside a 128-column record and inside a 256-column tile.  Logits against the oracle; decisions and
    every row statistic that does not depend on a summation order bit for bit against the 128 x 128
    tiles; the drafter's pass (arg-max only) likewise."""
    worst = 0.0
    for B, k, V in ((9, 4, 1000), (50, 5, 1000), (44, 6, 777), (37, 7, 300)):   # 45, 300, 308, 296 rows
        desc = synth.ModelDesc(0, 2, 128, 2, 256, V, 16, 64).resolved()
        case = cases.make_verify_case(desc, seed=900 + B, B=B, k=k, S=9, beta=3, tau=1.0, len_lo=0, len_hi=12,
                                      drafts="greedy", ragged_src=True, std=0.08)
        cases.run_oracle(case)
        tol = max(LOGIT_TOL, REL_TOL * float(case.logits.std()))
        outs = {}
        for name, opt in (("narrow", None), ("wide", {sd.SPECDEC_OPT_WIDE_VOCAB_TILES: 1})):
            ses = gh.open_verifier(case, options=opt)
            outs[name] = gh.gpu_verify(ses, case)
            ses.close()
            err = float(np.abs(outs[name]["logits"] - case.logits).max())
            worst = max(worst, err)
            assert err <= tol, (name, B, k, V, err)
            assert not cases.compare_decisions(case, outs[name]["accept"], outs[name]["next"])[2], (name, B, k, V)
        n, w = outs["narrow"], outs["wide"]
        assert np.array_equal(n["logits"], w["logits"]), (B, k, V)          # same MFMA chain per element
        assert np.array_equal(n["accept"], w["accept"]) and np.array_equal(n["next"], w["next"])
        for col in (0, 1, 3, 4):                                            # max, arg-max, z_d, count
            assert np.array_equal(n["stats"][..., col], w["stats"][..., col]), (B, k, V, col)
        assert np.abs(n["stats"][..., 2] - w["stats"][..., 2]).max() <= 1e-5, (B, k, V)   # log-sum-exp
        # the draft's logit is the logit of its column, bit for bit, in the wide kernel as well
        d = case.drafts
        zd = np.take_along_axis(w["logits"][:, :k, :], d[:, :, None].astype(np.int64), axis=2)[..., 0]
        assert np.array_equal(zd, w["stats"][:, :k, 3]), (B, k, V)
    print(f"[wide vocabulary tiles] worst max-abs logit err {worst:.3e}")


def test_wide_vocabulary_tiles_in_the_drafter_pass():
    """The drafter's pass on 256 x 256 tiles (records with max / arg-max only when no logits are asked
    for): slot logits, statistics, drafts and appended K/V against the oracle, 280 slot rows."""
    _, (dd, db, dm) = dl.make_models(seed=12)
    lens = synth.random_lengths(13, "len", 40, 0, 20)
    wz, wkv, ex = drafter_pass_case(dd, db, dm, B=40, S_max=13, k=7, lens=lens, seed=13, prefill=True, max_tgt=48,
                                    sample=(0, 7, 19, 39), options={sd.SPECDEC_OPT_WIDE_VOCAB_TILES: 1})
    print(f"[drafter, wide vocabulary tiles] logits max-abs err {wz:.3e}, K/V {wkv:.3e}, {ex} near-ties excused")


def test_random_medium_shapes_general_kernels():
    """Eight seeded random cases of 40-450 rows (batch 12-90, block size 1-15, prefixes 0-45, ragged
    sources of up to 40 tokens): the general kernels (64 x 64 and 128 x 128 GEMM tiles, one or two query
    tiles per attention wave, both vocabulary kernels, LayerNorm folded or as a pass of its own) against
    the oracle on every sequence."""
    desc = synth.ModelDesc(0, 2, 128, 2, 256, 1000, 40, 64).resolved()
    rng = np.random.default_rng(77)
    worst = 0.0
    for case_no in range(8):
        B = int(rng.integers(12, 91))
        k = int(rng.integers(max(1, 33 // B), 16))
        while B * (k + 1) <= 32:
            k += 1
        hi = int(rng.integers(0, 46))
        S = int(rng.integers(1, 41))
        case = cases.make_verify_case(desc, seed=700 + case_no, B=B, k=k, S=S, beta=int(rng.integers(1, 6)),
                                      tau=float(rng.choice([0.0, 0.5, 1.0, 3.0])), len_lo=0, len_hi=hi,
                                      drafts="greedy", ragged_src=True, std=0.08)
        cases.run_oracle(case)
        tol = max(LOGIT_TOL, REL_TOL * float(case.logits.std()))
        opt = {sd.SPECDEC_OPT_WIDE_VOCAB_TILES: case_no & 1, sd.SPECDEC_OPT_LN_FOLD: (case_no >> 1) & 1}
        ses = gh.open_verifier(case, options=opt)
        out = gh.gpu_verify(ses, case)
        ses.close()
        err = float(np.abs(out["logits"] - case.logits).max())
        worst = max(worst, err)
        assert err <= tol, (case_no, B, k, hi, S, opt, err)
        assert not cases.compare_decisions(case, out["accept"], out["next"])[2], (case_no, B, k, opt)
    print(f"[random medium shapes] 8 cases, worst max-abs logit err {worst:.3e}")


def test_kernel_kind_timing_counts_and_leaves_results_alone():
    """specdec_profile_select / specdec_profile_read: the number of timed launches per kind is the number the
    pass makes (3 residual-sum projections, 2 attentions, 1 QKV projection per layer, one vocabulary kernel),
    every duration is positive and small, for the kernels timed by their own begin / end (general kernels) and
    for those bracketed on the stream (small-batch kernels), and timing changes no result."""
    for B, k in ((40, 4), (5, 4)):                      # general kernels / fused small-batch kernels
        case = small_case(seed=61, B=B, k=k)
        ses = gh.open_verifier(case)
        ref = gh.gpu_verify(ses, case)
        Ld = case.desc.dec_layers
        for kind, per_pass in ((0, 3 * Ld), (3, 2 * Ld), (2, Ld), (4, 1)):
            sd.specdec_profile_select(ses.ctx, kind)
            sd.specdec_rewind(ses.ctx, ses.i32(case.lens))
            out = gh.gpu_verify(ses, case)
            ms, n = sd.specdec_profile_read(ses.ctx)
            if B * (k + 1) > 32:
                assert n == per_pass, (B, kind, n, per_pass)
            elif kind in (0, 4):                         # the fused kernels: attention runs inside kind 0
                assert n >= 1, (B, kind, n)
            assert n == 0 or 0.0 < ms < 5.0 * n, (B, kind, ms, n)
            assert np.array_equal(out["logits"], ref["logits"]) and np.array_equal(out["accept"], ref["accept"])
        sd.specdec_profile_select(ses.ctx, -1)
        ms, n = sd.specdec_profile_read(ses.ctx)
        assert n == 0
        ses.close()
