"""Shared test helpers: adapters between the synthetic-input module and the oracle."""
import numpy as np

from oracle import spts_oracle as orc
from paper_2601_13155_amd import synth


def oracle_model(shape: synth.ModelShape) -> orc.Model:
    return orc.Model(D=shape.D, H=shape.H, Hkv=shape.Hkv, d=shape.d, Dff=shape.Dff,
                     rms_eps=shape.rms_eps, rope_base=shape.rope_base)


def small_shape(dtype="f32", **kw) -> synth.ModelShape:
    base = dict(D=64, H=4, Hkv=2, d=16, Dff=96, rms_eps=1e-5, rope_base=10000.0, dtype=dtype)
    base.update(kw)
    return synth.ModelShape(**base)
