"""Seeded synthetic inputs for the SpecDec hot path (weights, memories, tokens).

This module only *draws* data: it holds none of the method's arithmetic and is
the single piece of code that both the CPU oracle's tests and the HIP path's
harness use, so that the two sides see the same numbers.  It depends on NumPy
only and never touches the GPU library.

The paper trains on WMT14/16 and CNN-DM with a joint 32K BPE dictionary and a
Transformer-base target model (Sec. 4.1, "Datasets and Evaluation", "Model
Configuration"); none of that data exists here, so every tensor is random with
the paper's *shapes*: vocabulary 32768, d_model/FFN 512/2048 (base) or
1024/4096 (big), 6+6 layers for the verifier and 12+2 for the Spec-Drafter.

Storage format of one model (this is the tensor order the C-ABI expects):
all tensors are bf16, matrices are ``[out_features, in_features]`` row-major
(``y = x @ W.T + b``), fused projections stack q, k, v (or k, v) along the
output axis.
"""
from __future__ import annotations

import zlib
from dataclasses import dataclass, asdict
from typing import Dict, List, Tuple

import numpy as np


@dataclass(frozen=True)
class ModelDesc:
    enc_layers: int
    dec_layers: int
    d_model: int
    n_heads: int
    d_ffn: int
    vocab: int
    max_src: int
    max_tgt: int
    bos_id: int = 0
    pad_id: int = 1
    eos_id: int = 2
    mask_id: int = -1          # -1 -> vocab - 1

    def resolved(self) -> "ModelDesc":
        if self.mask_id >= 0:
            return self
        d = asdict(self)
        d["mask_id"] = self.vocab - 1
        return ModelDesc(**d)


def base_verifier(max_src=128, max_tgt=128, enc_layers=6, vocab=32768) -> ModelDesc:
    return ModelDesc(enc_layers, 6, 512, 8, 2048, vocab, max_src, max_tgt).resolved()


def big_verifier(max_src=128, max_tgt=128, enc_layers=6, vocab=32768) -> ModelDesc:
    return ModelDesc(enc_layers, 6, 1024, 16, 4096, vocab, max_src, max_tgt).resolved()


def spec_drafter(max_src=128, max_tgt=128, enc_layers=12, vocab=32768) -> ModelDesc:
    return ModelDesc(enc_layers, 2, 512, 8, 2048, vocab, max_src, max_tgt).resolved()


# --------------------------------------------------------------------------- bf16
def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """Round-to-nearest-even fp32 -> bf16, returned as uint16 bit patterns."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    r = ((u >> np.uint32(16)) & np.uint32(1)) + np.uint32(0x7FFF)
    return ((u + r) >> np.uint32(16)).astype(np.uint16)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    return (b.astype(np.uint32) << np.uint32(16)).view(np.float32)


def round_bf16(x: np.ndarray) -> np.ndarray:
    """fp32 values rounded to the nearest bf16, still stored as fp32."""
    return bf16_bits_to_f32(f32_to_bf16_bits(x))


# --------------------------------------------------------------------------- streams
def stream(seed: int, name: str) -> np.random.Generator:
    """Independent named random stream: the draw for one tensor does not depend on
    which other tensors were drawn before it."""
    return np.random.default_rng([int(seed), zlib.crc32(name.encode())])


# --------------------------------------------------------------------------- weights
def tensor_specs(desc: ModelDesc) -> List[Tuple[str, Tuple[int, ...], str]]:
    """(name, shape, kind) in ABI order.  kind: 'w' matrix/bias ~N(0,0.02),
    'g' LayerNorm gain 1+N(0,0.02)."""
    d, f, v = desc.d_model, desc.d_ffn, desc.vocab
    out: List[Tuple[str, Tuple[int, ...], str]] = [("embed", (v, d), "w")]

    def ln(p):
        return [(p + ".g", (d,), "g"), (p + ".b", (d,), "w")]

    def ffn(p):
        return [(p + ".w1", (f, d), "w"), (p + ".b1", (f,), "w"),
                (p + ".w2", (d, f), "w"), (p + ".b2", (d,), "w")]

    for l in range(desc.enc_layers):
        p = f"enc.{l}"
        out += [(p + ".attn.wqkv", (3 * d, d), "w"), (p + ".attn.bqkv", (3 * d,), "w"),
                (p + ".attn.wo", (d, d), "w"), (p + ".attn.bo", (d,), "w")]
        out += ln(p + ".ln1") + ffn(p + ".ffn") + ln(p + ".ln2")
    for l in range(desc.dec_layers):
        p = f"dec.{l}"
        out += [(p + ".self.wqkv", (3 * d, d), "w"), (p + ".self.bqkv", (3 * d,), "w"),
                (p + ".self.wo", (d, d), "w"), (p + ".self.bo", (d,), "w")]
        out += ln(p + ".ln1")
        out += [(p + ".cross.wq", (d, d), "w"), (p + ".cross.bq", (d,), "w"),
                (p + ".cross.wkv", (2 * d, d), "w"), (p + ".cross.bkv", (2 * d,), "w"),
                (p + ".cross.wo", (d, d), "w"), (p + ".cross.bo", (d,), "w")]
        out += ln(p + ".ln2") + ffn(p + ".ffn") + ln(p + ".ln3")
    return out


def make_weights(desc: ModelDesc, seed: int, tag: str = "model", std: float = 0.02) -> Dict[str, np.ndarray]:
    """name -> uint16 bf16 bit patterns, in ABI order (dicts keep insertion order).
    std = 0.02 is the workload's init; small test models pass a larger std so that
    attention and LayerNorm are far from their trivial regimes."""
    out: Dict[str, np.ndarray] = {}
    for name, shape, kind in tensor_specs(desc):
        g = stream(seed, f"{tag}/{name}")
        x = g.standard_normal(shape, dtype=np.float32) * np.float32(std)
        if kind == "g":
            x = x + np.float32(1.0)
        out[name] = f32_to_bf16_bits(x)
    return out


def make_head_weights(desc: ModelDesc, n_heads: int, seed: int, std: float = 0.02) -> List[Dict[str, np.ndarray]]:
    """Drafting heads on top of a model (residual FFN blocks of the model's widths): per head
    w1 [F,d], b1 [F], w2 [d,F], b2 [d] as bf16 bit patterns."""
    d, f = desc.d_model, desc.d_ffn
    out = []
    for i in range(n_heads):
        hd = {}
        for name, shape in (("w1", (f, d)), ("b1", (f,)), ("w2", (d, f)), ("b2", (d,))):
            g = stream(seed, f"head{i}/{name}")
            hd[name] = f32_to_bf16_bits(g.standard_normal(shape, dtype=np.float32) * np.float32(std))
        out.append(hd)
    return out


def weights_f32(bits: Dict[str, np.ndarray]) -> Dict[str, np.ndarray]:
    return {k: bf16_bits_to_f32(v) for k, v in bits.items()}


# --------------------------------------------------------------------------- data
def make_memory(seed: int, B: int, S: int, d: int, name="memory") -> np.ndarray:
    """Encoder memory ~N(0,1), rounded to bf16 (returned as fp32 values) [B,S,d]."""
    g = stream(seed, name)
    return round_bf16(g.standard_normal((B, S, d), dtype=np.float32))


def random_tokens(seed: int, name: str, shape, desc: ModelDesc, full_vocab=False) -> np.ndarray:
    """'Uniform-random tokens': ordinary ids [4, V-2] (no special ids), or the whole
    vocabulary [0, V) when full_vocab (used for random drafts)."""
    g = stream(seed, name)
    if full_vocab:
        return g.integers(0, desc.vocab, size=shape, dtype=np.int64).astype(np.int32)
    return g.integers(4, desc.vocab - 1, size=shape, dtype=np.int64).astype(np.int32)


def random_lengths(seed: int, name: str, B: int, lo: int, hi: int) -> np.ndarray:
    """Integer lengths uniform in [lo, hi] inclusive."""
    g = stream(seed, name)
    return g.integers(lo, hi + 1, size=(B,), dtype=np.int64).astype(np.int32)


def corrupt(seed: int, name: str, tokens: np.ndarray, p: float, desc: ModelDesc) -> np.ndarray:
    """Replace each position independently with a uniform-random token w.p. p."""
    g = stream(seed, name)
    hit = g.random(tokens.shape) < p
    repl = g.integers(0, desc.vocab, size=tokens.shape, dtype=np.int64).astype(np.int32)
    return np.where(hit, repl, tokens).astype(np.int32)
