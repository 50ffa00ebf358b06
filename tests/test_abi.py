"""Host-side checks of the C ABI: the library loads, exports every entry point the header
declares, and validates arguments.  No kernel is launched here."""
import ctypes as C
import os
import re

import pytest

from paper_2203_16487_amd import binding as sd
from paper_2203_16487_amd import synth

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_library_exports_every_declared_symbol():
    hdr = open(os.path.join(ROOT, "include", "specdec.h")).read()
    hdr = re.sub(r"/\*.*?\*/", "", hdr, flags=re.S)
    declared = set(re.findall(r"\b(specdec_[a-z_]+)\s*\(", hdr))
    assert declared, "header parse failed"
    L = sd.lib()
    for name in declared:
        assert hasattr(L, name), f"{name} declared in specdec.h but not exported"
    assert declared == set(sd.EXPORTS), declared ^ set(sd.EXPORTS)


def test_weight_table_matches_input_generator():
    for desc in (synth.base_verifier(), synth.big_verifier(enc_layers=0), synth.spec_drafter()):
        specs = synth.tensor_specs(desc)
        assert sd.specdec_num_weights(desc) == len(specs)
        for i, (_, shape, _) in enumerate(specs):
            r, c = sd.specdec_weight_shape(desc, i)
            assert (r, c) == (shape[0], shape[1] if len(shape) > 1 else 1), (i, specs[i])


def test_create_rejects_bad_limits():
    for lim in [(0, 5, 8, 8), (4, 0, 8, 8), (4, 32, 8, 8), (4, 5, 0, 8), (4, 5, 8, 0)]:
        with pytest.raises(sd.SpecDecError) as e:
            sd.specdec_create(*lim)
        assert e.value.code == sd.SPECDEC_ERR_INVALID_ARG


def test_sizes_and_call_order_errors():
    ctx = sd.specdec_create(4, 10, 64, 64)
    try:
        assert sd.specdec_state_bytes(ctx) % 256 == 0 and sd.specdec_state_bytes(ctx) > 0
        small, big = synth.base_verifier(enc_layers=0), synth.big_verifier(enc_layers=0)
        ws, wb = sd.specdec_workspace_bytes(ctx, small), sd.specdec_workspace_bytes(ctx, big)
        assert 0 < ws < wb
        # KV arenas alone: 2 * Ld * B * (max_tgt + k_max + 1) * d * 2 bytes
        assert ws >= 2 * 6 * 4 * (64 + 10 + 1) * 512 * 2
        bad = synth.ModelDesc(0, 6, 500, 8, 2048, 32768, 64, 64).resolved()   # d != 64 * heads
        with pytest.raises(sd.SpecDecError) as e:
            sd.specdec_workspace_bytes(ctx, bad)
        assert e.value.code == sd.SPECDEC_ERR_INVALID_ARG
        L = sd.lib()
        # nothing bound yet
        assert L.specdec_begin(ctx, 1, 8, None) == sd.SPECDEC_ERR_BAD_STATE
        assert b"state" in L.specdec_last_error(ctx)
        assert L.specdec_verify(ctx, None, 5, 3, 1.0, None, None, None, None) == sd.SPECDEC_ERR_BAD_STATE
        assert L.specdec_commit(ctx, None, None, None, None) == sd.SPECDEC_ERR_BAD_STATE
        assert L.specdec_bind_state(ctx, None, 0) == sd.SPECDEC_ERR_INVALID_ARG
        assert L.specdec_bind_state(ctx, C.c_void_p(256), 16) == sd.SPECDEC_ERR_TOO_LARGE
        # null context
        assert L.specdec_begin(None, 1, 8, None) == sd.SPECDEC_ERR_INVALID_ARG
        assert L.specdec_last_error(None) == b"null context"
    finally:
        sd.specdec_destroy(ctx)


def test_bind_model_argument_checks_without_gpu():
    """bind_model validates before touching the device; with a fake (never dereferenced)
    pointer table it must fail on the count / alignment checks, or report NO_DEVICE."""
    ctx = sd.specdec_create(2, 5, 8, 8)
    try:
        L = sd.lib()
        desc = synth.ModelDesc(0, 1, 64, 1, 64, 64, 8, 8).resolved()
        n = sd.specdec_num_weights(desc)
        d = sd.make_desc(desc)
        ptrs = (C.c_void_p * n)(*[4096 + 16 * i for i in range(n)])
        assert L.specdec_bind_model(ctx, 0, C.byref(d), ptrs, n - 1, C.c_void_p(4096), 1 << 40, None) == sd.SPECDEC_ERR_INVALID_ARG
        assert L.specdec_bind_model(ctx, 7, C.byref(d), ptrs, n, C.c_void_p(4096), 1 << 40, None) == sd.SPECDEC_ERR_INVALID_ARG
        ptrs[3] = 4097
        assert L.specdec_bind_model(ctx, 0, C.byref(d), ptrs, n, C.c_void_p(4096), 1 << 40, None) == sd.SPECDEC_ERR_INVALID_ARG
        ptrs[3] = 4096
        assert L.specdec_bind_model(ctx, 0, C.byref(d), ptrs, n, C.c_void_p(4096), 16, None) == sd.SPECDEC_ERR_TOO_LARGE
        import torch
        if not torch.cuda.is_available():
            assert L.specdec_bind_model(ctx, 0, C.byref(d), ptrs, n, C.c_void_p(4096), 1 << 40, None) == sd.SPECDEC_ERR_NO_DEVICE
    finally:
        sd.specdec_destroy(ctx)


def test_bench_refuses_more_than_one_gpu():
    """bench.py --gpus N with N > 1 exits with a message (this build is one-GPU only)."""
    import subprocess
    import sys
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    r = subprocess.run([sys.executable, os.path.join(root, "bench.py"), "--gpus", "2"], capture_output=True, text=True)
    assert r.returncode == 2 and "ONE GPU" in r.stderr


def test_options_and_new_entry_points_validate_their_arguments():
    """specdec_configure, the FP8 workspace sizing, specdec_quantize_rows, specdec_bind_draft_heads and
    specdec_verify_static: argument checks that need no GPU."""
    ctx = sd.specdec_create(4, 10, 64, 64)
    try:
        L = sd.lib()
        assert L.specdec_configure(ctx, 99, 1) == sd.SPECDEC_ERR_INVALID_ARG
        assert L.specdec_configure(ctx, sd.SPECDEC_OPT_RESIDENT, 2) == sd.SPECDEC_ERR_INVALID_ARG
        assert L.specdec_configure(None, sd.SPECDEC_OPT_RESIDENT, 1) == sd.SPECDEC_ERR_INVALID_ARG
        assert L.specdec_configure(ctx, sd.SPECDEC_OPT_WIDE_VOCAB_TILES, 2) == sd.SPECDEC_ERR_INVALID_ARG
        assert L.specdec_configure(ctx, sd.SPECDEC_OPT_WIDE_VOCAB_TILES, 1) == sd.SPECDEC_OK
        assert L.specdec_configure(ctx, sd.SPECDEC_OPT_WIDE_VOCAB_TILES, 0) == sd.SPECDEC_OK
        desc = synth.base_verifier(enc_layers=0)
        d, F, V, Ld = desc.d_model, desc.d_ffn, desc.vocab, desc.dec_layers
        w0 = sd.specdec_workspace_bytes(ctx, desc)
        sd.specdec_configure(ctx, sd.SPECDEC_OPT_FP8_WEIGHTS, 1)
        w1 = sd.specdec_workspace_bytes(ctx, desc)
        # one byte per weight of the six decoder matrices and of the output matrix, one fp32 scale per row
        extra = Ld * (6 * d * d + 2 * d * F) + V * d + 4 * (Ld * (7 * d + F) + V)
        assert extra <= w1 - w0 <= extra + 4096
        sd.specdec_configure(ctx, sd.SPECDEC_OPT_FP8_CROSS_KV, 1)
        w2 = sd.specdec_workspace_bytes(ctx, desc)
        # codes for keys and values + their scales: (1 + 1 + 2 * 4 / 64) bytes per element of one bf16 arena
        arena = Ld * 4 * desc.n_heads * 64 * 64          # layers x max_batch x heads x Scap(64) x 64
        assert 2 * arena + 2 * arena // 16 <= w2 - w1 <= 2 * arena + 2 * arena // 16 + 4096
        sd.specdec_configure(ctx, sd.SPECDEC_OPT_FP8_WEIGHTS, 0)
        sd.specdec_configure(ctx, sd.SPECDEC_OPT_FP8_CROSS_KV, 0)
        assert sd.specdec_workspace_bytes(ctx, desc) == w0
        one = C.c_void_p(16)
        assert L.specdec_quantize_rows(ctx, None, 4, 64, one, one, None) == sd.SPECDEC_ERR_INVALID_ARG
        assert L.specdec_quantize_rows(ctx, one, 4, 60, one, one, None) == sd.SPECDEC_ERR_INVALID_ARG     # K % 8
        assert L.specdec_quantize_rows(ctx, one, -1, 64, one, one, None) == sd.SPECDEC_ERR_INVALID_ARG
        assert L.specdec_quantize_rows(ctx, C.c_void_p(8), 4, 64, one, one, None) == sd.SPECDEC_ERR_INVALID_ARG  # alignment
        assert b"aligned" in L.specdec_last_error(ctx)
        # nothing bound yet: the hot-path variants refuse, and say why
        assert L.specdec_verify_static(ctx, None, 5, 3, 1.0, None, None, None, None) == sd.SPECDEC_ERR_BAD_STATE
        assert L.specdec_draft_heads(ctx, None, 3, None, None, None) == sd.SPECDEC_ERR_BAD_STATE
        assert L.specdec_bind_draft_heads(ctx, 3, None, None, None, None) != sd.SPECDEC_OK
    finally:
        sd.specdec_destroy(ctx)
