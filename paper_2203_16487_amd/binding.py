"""ctypes binding of libspecdec.so: same names as include/specdec.h, argument
marshalling only.  Every step of the path runs in the library's HIP kernels;
PyTorch appears here only as the owner of device memory and streams.

The library must have been built (python -m paper_2203_16487_amd.build); there
is no fallback of any kind: a missing library raises.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import Dict, Optional, Sequence

import numpy as np

HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(HERE, "libspecdec.so")

SPECDEC_OK = 0
SPECDEC_ERR_INVALID_ARG = -1
SPECDEC_ERR_BAD_STATE = -2
SPECDEC_ERR_TOO_LARGE = -3
SPECDEC_ERR_HIP = -4
SPECDEC_ERR_NO_DEVICE = -5
SPECDEC_VERIFIER = 0
SPECDEC_DRAFTER = 1
SPECDEC_ROW_STATS = 8
ROW_STATS = SPECDEC_ROW_STATS
SPECDEC_COUNTERS = 8
SPECDEC_OPT_SMALL_BATCH_KERNELS = 0
SPECDEC_OPT_LN_FOLD = 1
SPECDEC_OPT_RESIDENT = 2
SPECDEC_OPT_SLICED_SUBLAYERS = 3
SPECDEC_OPT_FP8_WEIGHTS = 4
SPECDEC_OPT_FP8_CROSS_KV = 5
SPECDEC_OPT_WIDE_VOCAB_TILES = 6


class specdec_model_desc(C.Structure):
    _fields_ = [(n, C.c_int32) for n in ("enc_layers", "dec_layers", "d_model", "n_heads", "d_ffn", "vocab",
                                         "bos_id", "eos_id", "pad_id", "mask_id")]


class specdec_limits(C.Structure):
    _fields_ = [(n, C.c_int32) for n in ("max_batch", "k_max", "max_src", "max_tgt")]


EXPORTS = {
    "specdec_create": (C.c_int, [C.POINTER(C.c_void_p), C.POINTER(specdec_limits)]),
    "specdec_destroy": (None, [C.c_void_p]),
    "specdec_last_error": (C.c_char_p, [C.c_void_p]),
    "specdec_num_weights": (C.c_int, [C.POINTER(specdec_model_desc), C.POINTER(C.c_int32)]),
    "specdec_weight_shape": (C.c_int, [C.POINTER(specdec_model_desc), C.c_int32, C.POINTER(C.c_int64), C.POINTER(C.c_int64)]),
    "specdec_state_bytes": (C.c_int, [C.c_void_p, C.POINTER(C.c_size_t)]),
    "specdec_bind_state": (C.c_int, [C.c_void_p, C.c_void_p, C.c_size_t]),
    "specdec_workspace_bytes": (C.c_int, [C.c_void_p, C.POINTER(specdec_model_desc), C.POINTER(C.c_size_t)]),
    "specdec_bind_model": (C.c_int, [C.c_void_p, C.c_int, C.POINTER(specdec_model_desc), C.POINTER(C.c_void_p),
                                     C.c_int32, C.c_void_p, C.c_size_t, C.c_void_p]),
    "specdec_begin": (C.c_int, [C.c_void_p, C.c_int32, C.c_int32, C.c_void_p]),
    "specdec_encode": (C.c_int, [C.c_void_p, C.c_void_p, C.c_void_p, C.c_int32, C.c_void_p]),
    "specdec_set_memory": (C.c_int, [C.c_void_p, C.c_int, C.c_void_p, C.c_void_p, C.c_int32, C.c_void_p]),
    "specdec_set_stream": (C.c_int, [C.c_void_p, C.c_void_p, C.c_void_p, C.c_int32, C.c_void_p]),
    "specdec_load_cache": (C.c_int, [C.c_void_p, C.c_int, C.c_void_p, C.c_void_p, C.c_void_p, C.c_int32, C.c_void_p]),
    "specdec_prefill": (C.c_int, [C.c_void_p, C.c_int, C.c_void_p]),
    "specdec_draft": (C.c_int, [C.c_void_p, C.c_int32, C.c_void_p, C.c_void_p, C.c_void_p]),
    "specdec_bind_draft_heads": (C.c_int, [C.c_void_p, C.c_int32, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p]),
    "specdec_draft_heads": (C.c_int, [C.c_void_p, C.c_void_p, C.c_int32, C.c_void_p, C.c_void_p, C.c_void_p]),
    "specdec_configure": (C.c_int, [C.c_void_p, C.c_int32, C.c_int32]),
    "specdec_set_prefix": (C.c_int, [C.c_void_p, C.c_int, C.c_void_p, C.c_void_p, C.c_int32, C.c_void_p, C.c_void_p, C.c_void_p]),
    "specdec_get_draft_stats": (C.c_int, [C.c_void_p, C.c_void_p, C.c_void_p]),
    "specdec_get_counters": (C.c_int, [C.c_void_p, C.c_void_p, C.c_void_p]),
    "specdec_quantize_rows": (C.c_int, [C.c_void_p, C.c_void_p, C.c_int64, C.c_int64, C.c_void_p, C.c_void_p,
                                             C.c_void_p]),
    "specdec_verify": (C.c_int, [C.c_void_p, C.c_void_p, C.c_int32, C.c_int32, C.c_float, C.c_void_p, C.c_void_p,
                                 C.c_void_p, C.c_void_p]),
    "specdec_verify_static": (C.c_int, [C.c_void_p, C.c_void_p, C.c_int32, C.c_int32, C.c_float, C.c_void_p, C.c_void_p,
                                        C.c_void_p, C.c_void_p]),
    "specdec_commit": (C.c_int, [C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p]),
    "specdec_rewind": (C.c_int, [C.c_void_p, C.c_void_p, C.c_void_p]),
    "specdec_profile_select": (C.c_int, [C.c_void_p, C.c_int32]),
    "specdec_profile_read": (C.c_int, [C.c_void_p, C.POINTER(C.c_double), C.POINTER(C.c_int32)]),
    "specdec_get_output": (C.c_int, [C.c_void_p, C.c_void_p, C.c_int32, C.c_void_p, C.c_void_p, C.c_void_p]),
    "specdec_get_cache": (C.c_int, [C.c_void_p, C.c_int, C.c_void_p, C.c_void_p, C.c_int32, C.c_void_p]),
    "specdec_get_row_stats": (C.c_int, [C.c_void_p, C.c_void_p, C.c_void_p]),
    "specdec_get_memory": (C.c_int, [C.c_void_p, C.c_int, C.c_void_p, C.c_void_p]),
}

_lib = None


def lib() -> C.CDLL:
    """The loaded library; raises if it has not been built."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError(f"{LIB_PATH} is missing: run `python -m paper_2203_16487_amd.build` "
                               "(there is no fallback path)")
        # PyTorch owns the device memory this binding hands over, so both must talk to ONE HIP
        # runtime: importing torch first makes its libamdhip64 the one libspecdec binds to
        # (two runtimes in one process do not see the GPU).
        import torch  # noqa: F401
        L = C.CDLL(LIB_PATH)
        for name, (res, args) in EXPORTS.items():
            f = getattr(L, name)
            f.restype, f.argtypes = res, args
        _lib = L
    return _lib


class SpecDecError(RuntimeError):
    def __init__(self, code: int, msg: str):
        super().__init__(f"libspecdec error {code}: {msg}")
        self.code = code


def _check(ctx, rc: int):
    if rc != SPECDEC_OK:
        msg = lib().specdec_last_error(ctx).decode() if ctx else "(no context)"
        raise SpecDecError(rc, msg)


def make_desc(d) -> specdec_model_desc:
    """From any object with the fields of specdec_model_desc (e.g. synth.ModelDesc)."""
    return specdec_model_desc(*[int(getattr(d, n)) for n, _ in specdec_model_desc._fields_])


def _ptr(t) -> Optional[int]:
    """Device pointer of a torch tensor (None -> NULL)."""
    if t is None:
        return None
    assert t.is_contiguous(), "tensors handed to libspecdec must be contiguous"
    return t.data_ptr()


def _stream() -> int:
    import torch
    return torch.cuda.current_stream().cuda_stream


# ------------------------------------------------------------------------ same-name wrappers
def specdec_create(max_batch: int, k_max: int, max_src: int, max_tgt: int) -> C.c_void_p:
    ctx = C.c_void_p()
    lim = specdec_limits(max_batch, k_max, max_src, max_tgt)
    rc = lib().specdec_create(C.byref(ctx), C.byref(lim))
    if rc != SPECDEC_OK:
        raise SpecDecError(rc, "specdec_create: bad limits")
    return ctx


def specdec_destroy(ctx):
    lib().specdec_destroy(ctx)


def specdec_num_weights(desc) -> int:
    n = C.c_int32()
    _check(None, lib().specdec_num_weights(C.byref(make_desc(desc)), C.byref(n)))
    return n.value


def specdec_weight_shape(desc, idx: int):
    r, c = C.c_int64(), C.c_int64()
    _check(None, lib().specdec_weight_shape(C.byref(make_desc(desc)), idx, C.byref(r), C.byref(c)))
    return r.value, c.value


def specdec_state_bytes(ctx) -> int:
    n = C.c_size_t()
    _check(ctx, lib().specdec_state_bytes(ctx, C.byref(n)))
    return n.value


def specdec_bind_state(ctx, buf):
    _check(ctx, lib().specdec_bind_state(ctx, _ptr(buf), buf.numel() * buf.element_size()))


def specdec_workspace_bytes(ctx, desc) -> int:
    n = C.c_size_t()
    _check(ctx, lib().specdec_workspace_bytes(ctx, C.byref(make_desc(desc)), C.byref(n)))
    return n.value


def specdec_bind_model(ctx, role: int, desc, weights: Sequence, workspace):
    arr = (C.c_void_p * len(weights))(*[_ptr(w) for w in weights])
    _check(ctx, lib().specdec_bind_model(ctx, role, C.byref(make_desc(desc)), arr, len(weights), _ptr(workspace),
                                         workspace.numel() * workspace.element_size(), _stream()))


def specdec_begin(ctx, B: int, max_new: int):
    _check(ctx, lib().specdec_begin(ctx, B, max_new, _stream()))


def specdec_encode(ctx, src, src_len):
    _check(ctx, lib().specdec_encode(ctx, _ptr(src), _ptr(src_len), src.shape[1], _stream()))


def specdec_set_memory(ctx, role: int, memory, src_len):
    _check(ctx, lib().specdec_set_memory(ctx, role, _ptr(memory), _ptr(src_len), memory.shape[1], _stream()))


def specdec_set_stream(ctx, tokens, length):
    _check(ctx, lib().specdec_set_stream(ctx, _ptr(tokens), _ptr(length), tokens.shape[1] - 1, _stream()))


def specdec_load_cache(ctx, role: int, k_cache, v_cache, n):
    _check(ctx, lib().specdec_load_cache(ctx, role, _ptr(k_cache), _ptr(v_cache), _ptr(n), k_cache.shape[2], _stream()))


def specdec_prefill(ctx, role: int):
    _check(ctx, lib().specdec_prefill(ctx, role, _stream()))


def specdec_draft(ctx, k: int, draft, logits=None):
    _check(ctx, lib().specdec_draft(ctx, k, _ptr(draft), _ptr(logits), _stream()))


def specdec_bind_draft_heads(ctx, n_heads: int, w1, b1, w2, b2):
    _check(ctx, lib().specdec_bind_draft_heads(ctx, n_heads, _ptr(w1), _ptr(b1), _ptr(w2), _ptr(b2)))


def specdec_draft_heads(ctx, accept_len, k: int, draft, logits=None):
    _check(ctx, lib().specdec_draft_heads(ctx, _ptr(accept_len), k, _ptr(draft), _ptr(logits), _stream()))


def specdec_configure(ctx, option: int, value: int):
    _check(ctx, lib().specdec_configure(ctx, option, value))


def specdec_set_prefix(ctx, role: int, tokens, length, k_cache, v_cache):
    _check(ctx, lib().specdec_set_prefix(ctx, role, _ptr(tokens), _ptr(length), tokens.shape[1] - 1, _ptr(k_cache),
                                         _ptr(v_cache), _stream()))


def specdec_get_draft_stats(ctx, stats):
    _check(ctx, lib().specdec_get_draft_stats(ctx, _ptr(stats), _stream()))


def specdec_get_counters(ctx, counters):
    _check(ctx, lib().specdec_get_counters(ctx, _ptr(counters), _stream()))


def specdec_quantize_rows(ctx, w, codes, scale):
    N, K = w.shape
    _check(ctx, lib().specdec_quantize_rows(ctx, _ptr(w), N, K, _ptr(codes), _ptr(scale), _stream()))


def specdec_verify(ctx, draft, k: int, beta: int, tau: float, accept_len, next_token, logits=None):
    _check(ctx, lib().specdec_verify(ctx, _ptr(draft), k, beta, tau, _ptr(accept_len), _ptr(next_token),
                                     _ptr(logits), _stream()))


def specdec_verify_static(ctx, draft, k: int, beta: int, tau: float, accept_len, next_token, logits=None):
    _check(ctx, lib().specdec_verify_static(ctx, _ptr(draft), k, beta, tau, _ptr(accept_len), _ptr(next_token),
                                            _ptr(logits), _stream()))


def specdec_commit(ctx, accept_len, next_token, n_active=None):
    _check(ctx, lib().specdec_commit(ctx, _ptr(accept_len), _ptr(next_token), _ptr(n_active), _stream()))


def specdec_rewind(ctx, length):
    _check(ctx, lib().specdec_rewind(ctx, _ptr(length), _stream()))


KIND = dict(none=-1, gemm_f32=0, gemm_bf16=1, gemm_qkv=2, attn=3, vocab=4, ln=5, accept=6, other=7, resident=8)


def specdec_profile_select(ctx, kind: int):
    _check(ctx, lib().specdec_profile_select(ctx, kind))


def specdec_profile_read(ctx):
    ms, n = C.c_double(), C.c_int32()
    _check(ctx, lib().specdec_profile_read(ctx, C.byref(ms), C.byref(n)))
    return ms.value, n.value


def specdec_get_output(ctx, tokens, out_len, finished=None):
    _check(ctx, lib().specdec_get_output(ctx, _ptr(tokens), tokens.shape[1], _ptr(out_len), _ptr(finished), _stream()))


def specdec_get_cache(ctx, role: int, k_cache, v_cache):
    _check(ctx, lib().specdec_get_cache(ctx, role, _ptr(k_cache), _ptr(v_cache), k_cache.shape[2], _stream()))


def specdec_get_memory(ctx, role: int, memory):
    _check(ctx, lib().specdec_get_memory(ctx, role, _ptr(memory), _stream()))


def specdec_get_row_stats(ctx, stats):
    _check(ctx, lib().specdec_get_row_stats(ctx, _ptr(stats), _stream()))


# ------------------------------------------------------------------------ device memory holder
class Session:
    """Owns the context and the torch tensors (weights, workspaces, state) it points into.
    Allocation and pointer marshalling only."""

    def __init__(self, max_batch: int, k_max: int, max_src: int, max_tgt: int, device="cuda:0", fill: int = 0):
        """fill: byte the state and workspace buffers hold before they are bound (the header lets the
        caller pass any buffer: 0xFF makes every untouched bf16 / fp32 word a NaN)."""
        import torch
        self.torch = torch
        self.device = torch.device(device)
        self.ctx = specdec_create(max_batch, k_max, max_src, max_tgt)
        self.limits = (max_batch, k_max, max_src, max_tgt)
        self._keep = []
        self.fill = int(fill)
        self.state = torch.full((specdec_state_bytes(self.ctx),), self.fill, dtype=torch.uint8, device=self.device)
        specdec_bind_state(self.ctx, self.state)
        self.desc: Dict[int, object] = {}

    def upload_weights(self, bits: Dict[str, np.ndarray]):
        """name -> uint16 bf16 bit patterns (ABI order) -> list of device bf16 tensors."""
        torch = self.torch
        out = []
        for v in bits.values():
            t = torch.from_numpy(np.ascontiguousarray(v).view(np.int16)).to(self.device).view(torch.bfloat16)
            out.append(t)
        return out

    def bind_model(self, role: int, desc, weights: Sequence):
        torch = self.torch
        ws = torch.full((specdec_workspace_bytes(self.ctx, desc),), self.fill, dtype=torch.uint8, device=self.device)
        specdec_bind_model(self.ctx, role, desc, weights, ws)
        self._keep.append((weights, ws))
        self.desc[role] = desc
        return ws

    def i32(self, a):
        return self.torch.as_tensor(np.ascontiguousarray(a, dtype=np.int32), device=self.device)

    def bf16(self, a_f32: np.ndarray):
        """fp32 array -> device bf16 tensor (round to nearest even)."""
        return self.torch.from_numpy(np.ascontiguousarray(a_f32, dtype=np.float32)).to(self.device).to(self.torch.bfloat16).contiguous()

    def close(self):
        if self.ctx is not None:
            self.torch.cuda.synchronize(self.device)
            specdec_destroy(self.ctx)
            self.ctx = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass
