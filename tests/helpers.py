"""Shared test helpers: tiny models for the oracle pins, case builders for parity."""
from __future__ import annotations

import numpy as np

from paper_2203_16487_amd import synth
import specdec_oracle as orc


def tiny_desc(enc_layers=2, dec_layers=2, d=32, H=4, F=64, V=50, max_src=16, max_tgt=24):
    return synth.ModelDesc(enc_layers, dec_layers, d, H, F, V, max_src, max_tgt).resolved()


def tiny_model(seed=0, dtype=np.float32, std=0.25, **kw) -> orc.Model:
    desc = tiny_desc(**kw)
    w = synth.weights_f32(synth.make_weights(desc, seed, std=std))
    return orc.Model(desc, {k: v.astype(dtype) for k, v in w.items()})


def tiny_memory(model, seed=0, S=7):
    return synth.make_memory(seed, 1, S, model.desc.d_model)[0].astype(model.dtype)


def prefilled_state(model, memory, prefix_tokens, cap):
    """Verifier state with K/V of prefix_tokens cached by sequential AR steps."""
    st = orc.new_state(model, memory, cap)
    for t in prefix_tokens:
        orc.dec_step(model, st, int(t))
    return st
