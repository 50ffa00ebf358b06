"""FP8 (E4M3, per-row scale) weight streaming for passes of at most 32 rows, through the C ABI.

Two bars.  The conversion itself is an encoding: codes and scales must equal the oracle's bit for
bit.  The pass that streams the codes is held to the same logit tolerance against the oracle's
QUANTISED model (the model whose matrices are scale * decode(code)) as the bf16 pass is against the
bf16 model: the codes are exact in bf16, so the only extra rounding is the fp32 product with the
row scale.  Against the bf16 model the quantised one differs by the format's error, which the last
test reports (it is a property of the format, not of the kernels)."""
import numpy as np
import pytest
import torch

import cases
import gpu_harness as gh
import specdec_oracle as orc
from paper_2203_16487_amd import binding as sd
from paper_2203_16487_amd import synth

pytestmark = pytest.mark.gpu
LOGIT_TOL = 2e-2
REL_TOL = 0.04
FP8 = {sd.SPECDEC_OPT_FP8_WEIGHTS: 1}


def test_quantiser_matches_the_oracle_bit_for_bit():
    rng = np.random.default_rng(5)
    ses = sd.Session(1, 1, 8, 8)
    for N, K, kind in ((37, 128, "normal"), (64, 1024, "normal"), (5, 4096, "wide"), (9, 64, "special")):
        w = rng.normal(0, 0.02, (N, K)).astype(np.float32)
        if kind == "wide":     # eight decades of magnitude in every row: subnormal codes and flushes to zero
            w *= np.exp(rng.uniform(-18, 0, (N, K))).astype(np.float32)
        if kind == "special":
            w[0] = 0.0                               # all-zero row: scale 1
            w[1, :] = 0.0; w[1, 3] = -1.5            # a single entry: it becomes -448
            w[2, :8] = [1, 0.5 + 1 / 32, 0.5 + 3 / 32, 2 ** -10, 2 ** -9, -1, 1 / 256, 1 / 1024]
        wb = synth.f32_to_bf16_bits(w)
        wf = synth.bf16_bits_to_f32(wb)
        codes_o, scale_o, _ = orc.quantize_rows_e4m3(wf)
        wt = torch.from_numpy(wb.view(np.int16)).to(ses.device).view(torch.bfloat16)
        codes = torch.full((N, K), 0xAA, dtype=torch.uint8, device=ses.device)
        scale = torch.full((N,), float("nan"), dtype=torch.float32, device=ses.device)
        sd.specdec_quantize_rows(ses.ctx, wt, codes, scale)
        torch.cuda.synchronize()
        assert np.array_equal(scale.cpu().numpy().view(np.uint32), scale_o.view(np.uint32)), (N, K, kind)
        bad = np.argwhere(codes.cpu().numpy() != codes_o)
        assert bad.size == 0, (N, K, kind, bad[:5])
    ses.close()


@pytest.mark.parametrize("shape", ["toy", "base_b1", "base_b3", "big_b1"])
def test_fp8_small_batch_pass_matches_the_quantised_oracle(shape):
    if shape == "toy":
        desc = synth.ModelDesc(0, 2, 128, 2, 256, 1000, 16, 64).resolved()
        args = dict(seed=81, B=5, S=9, k=4, len_lo=0, len_hi=14, std=0.08)
    elif shape == "base_b1":
        desc = synth.base_verifier(max_src=32, max_tgt=64, enc_layers=0)
        args = dict(seed=82, B=1, S=24, k=25, len_lo=17, len_hi=17, std=0.02)
    elif shape == "base_b3":
        desc = synth.base_verifier(max_src=32, max_tgt=64, enc_layers=0)
        args = dict(seed=83, B=3, S=24, k=9, len_lo=0, len_hi=20, std=0.02)
    else:   # d = 1024, F = 4096: the long-k FFN2 path that is not staged through LDS at 32 rows
        desc = synth.ModelDesc(0, 2, 1024, 16, 4096, 4099, 32, 64).resolved()
        args = dict(seed=84, B=1, S=20, k=30, len_lo=11, len_hi=11, std=0.02)
    case = cases.make_verify_case(desc, beta=3, tau=1.0, drafts="greedy", ragged_src=True, fp8=True, **args)
    cases.run_oracle(case)
    ses = gh.open_verifier(case, options=FP8)
    out = gh.gpu_verify(ses, case)
    L = case.L_max + case.k + 1
    Kg, Vg = gh.gpu_cache(ses, case, L)
    ses.close()
    err = float(np.abs(out["logits"] - case.logits).max())
    zstd = float(case.logits.std())
    print(f"[fp8 {shape}] logit std {zstd:.3f}, max-abs err vs the quantised oracle {err:.3e}")
    assert err <= max(LOGIT_TOL, REL_TOL * zstd)
    n_exact, n_excused, bad = cases.compare_decisions(case, out["accept"], out["next"])
    assert not bad, bad
    # the rows this pass appended to the cache
    for b, st in enumerate(case.states):
        j = int(case.lens[b])
        for l in range(desc.dec_layers):
            assert np.abs(Kg[l, b, j:j + case.k + 1] - st.K[l][j:j + case.k + 1]).max() <= 3e-2
            assert np.abs(Vg[l, b, j:j + case.k + 1] - st.V[l][j:j + case.k + 1]).max() <= 3e-2
    # row statistics agree with the logits this pass wrote (count, draft logit)
    z = out["logits"]
    for b in range(case.B):
        for i in range(case.k):
            zd = z[b, i, case.drafts[b, i]]
            assert out["stats"][b, i, 3] == zd
            assert int(out["stats"][b, i, 4]) == int((z[b, i] > zd).sum())


def test_fp8_is_refused_by_the_paths_that_do_not_stream_it_and_ignored_by_large_passes():
    desc = synth.ModelDesc(0, 2, 128, 2, 256, 1000, 16, 64).resolved()
    case = cases.make_verify_case(desc, seed=85, B=2, S=9, k=4, beta=3, tau=1.0, len_lo=3, len_hi=9, drafts="greedy",
                                  std=0.08, fp8=True)
    ses = gh.open_verifier(case, options={**FP8, sd.SPECDEC_OPT_RESIDENT: 1})
    with pytest.raises(sd.SpecDecError):
        gh.gpu_verify(ses, case)
    ses.close()
    # 40 rows: the general kernels, which read the bf16 matrices
    big = cases.make_verify_case(desc, seed=86, B=8, S=9, k=4, beta=3, tau=1.0, len_lo=3, len_hi=9, drafts="greedy",
                                 std=0.08)
    cases.run_oracle(big)
    ses = gh.open_verifier(big, options=FP8)
    out = gh.gpu_verify(ses, big)
    ses.close()
    zstd = float(big.logits.std())
    assert np.abs(out["logits"] - big.logits).max() <= max(LOGIT_TOL, REL_TOL * zstd)


def test_fp8_format_error_is_reported():
    """How far the quantised model is from the bf16 one (oracle against oracle would say the same;
    here both passes run on the GPU, same inputs, same cache)."""
    desc = synth.base_verifier(max_src=32, max_tgt=64, enc_layers=0)
    case = cases.make_verify_case(desc, seed=87, B=1, S=24, k=25, beta=3, tau=1.0, len_lo=9, len_hi=9, drafts="greedy",
                                  std=0.02)
    cases.run_oracle(case)
    outs = {}
    for name, opt in (("bf16", None), ("fp8", FP8)):
        ses = gh.open_verifier(case, options=opt)
        outs[name] = gh.gpu_verify(ses, case)
        ses.close()
    diff = float(np.abs(outs["fp8"]["logits"] - outs["bf16"]["logits"]).max())
    zstd = float(case.logits.std())
    same_top = float((outs["fp8"]["logits"].argmax(-1) == outs["bf16"]["logits"].argmax(-1)).mean())
    print(f"[fp8 format] max-abs logit change {diff:.3e} ({diff / zstd:.1%} of the logit std {zstd:.3f}), "
          f"same arg-max on {same_top:.0%} of rows")
    assert diff <= 0.5 * zstd     # E4M3's 2^-4 relative step per weight, averaged over d = 512 terms and six layers


# ----------------------------------------------------------------------------- FP8 cross-attention keys / values
KV8 = {sd.SPECDEC_OPT_FP8_CROSS_KV: 1}


@pytest.mark.parametrize("shape", ["toy_small", "toy_general", "toy_long_source", "base_b3", "both_formats", "garbage_fill"])
def test_fp8_cross_kv_matches_the_quantised_oracle(shape):
    """Cross keys / values stored as E4M3 with one scale per (key, head) vector, against the oracle whose
    state holds the same stored values.  The library converts from its bf16 arenas, the oracle from
    unrounded values: a code may differ by one step where bf16 rounding crosses an E4M3 boundary, which
    stays far inside the logit tolerance.  Cases: the fused small-batch kernels, the general kernels
    (40 rows), a source longer than 256 (4-way key split), the base verifier, both FP8 options at once,
    and buffers filled with 0xFF (dead keys then carry NaN codes AND NaN scales)."""
    toy = synth.ModelDesc(0, 2, 128, 2, 256, 1000, 16, 64).resolved()
    opts, fill, fp8w = dict(KV8), 0, False
    if shape == "toy_small":
        desc, args = toy, dict(seed=91, B=5, S=9, k=4, len_lo=0, len_hi=14, std=0.08)
    elif shape == "toy_general":
        desc, args = toy, dict(seed=92, B=8, S=40, k=4, len_lo=0, len_hi=14, std=0.08)
    elif shape == "toy_long_source":
        desc = synth.ModelDesc(0, 2, 128, 2, 256, 1000, 320, 64).resolved()
        args = dict(seed=93, B=3, S=300, k=4, len_lo=2, len_hi=9, std=0.08)
    elif shape == "base_b3":
        desc = synth.base_verifier(max_src=32, max_tgt=64, enc_layers=0)
        args = dict(seed=94, B=3, S=24, k=9, len_lo=0, len_hi=20, std=0.02)
    elif shape == "both_formats":
        desc = synth.base_verifier(max_src=32, max_tgt=64, enc_layers=0)
        args = dict(seed=95, B=1, S=32, k=5, len_lo=16, len_hi=16, std=0.02)
        opts.update(FP8)
        fp8w = True
    else:
        desc, args, fill = toy, dict(seed=96, B=5, S=9, k=4, len_lo=0, len_hi=14, std=0.08), 0xFF
    case = cases.make_verify_case(desc, beta=3, tau=1.0, drafts="greedy", ragged_src=True, fp8=fp8w, fp8_kv=True, **args)
    cases.run_oracle(case)
    ses = gh.open_verifier(case, options=opts, fill=fill)
    out = gh.gpu_verify(ses, case)
    ses.close()
    assert np.isfinite(out["logits"]).all()
    err = float(np.abs(out["logits"] - case.logits).max())
    zstd = float(case.logits.std())
    print(f"[fp8 cross-kv {shape}] logit std {zstd:.3f}, max-abs err vs the quantised oracle {err:.3e}")
    assert err <= max(LOGIT_TOL, REL_TOL * zstd)
    assert not cases.compare_decisions(case, out["accept"], out["next"])[2]


def test_fp8_cross_kv_format_error_is_reported():
    """Both passes on the GPU, same inputs: how far E4M3 keys / values move the logits of the bf16 model."""
    desc = synth.base_verifier(max_src=64, max_tgt=64, enc_layers=0)
    case = cases.make_verify_case(desc, seed=97, B=2, S=64, k=9, beta=3, tau=1.0, len_lo=9, len_hi=12, drafts="greedy",
                                  std=0.02)
    cases.run_oracle(case)
    outs = {}
    for name, opt in (("bf16", None), ("fp8", KV8)):
        ses = gh.open_verifier(case, options=opt)
        outs[name] = gh.gpu_verify(ses, case)
        ses.close()
    diff = float(np.abs(outs["fp8"]["logits"] - outs["bf16"]["logits"]).max())
    zstd = float(case.logits.std())
    print(f"[fp8 cross-kv format] max-abs logit change {diff:.3e} ({diff / zstd:.1%} of the logit std {zstd:.3f})")
    assert 0 < diff <= 0.25 * zstd
