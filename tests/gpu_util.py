"""Helpers shared by the GPU parity tests: the same seeded inputs go to both sides."""
import numpy as np

import synth
from oracle import transformer as otf


def oracle_model(shape, seed=0, unit_gains=False, head=True, cache=True):
    hw = synth.head_weights(shape, seed, unit_gains) if head else None
    return otf.Model(shape, lambda l: synth.layer_weights(shape, l, seed, unit_gains), hw, cache=cache)


def gpu_engine(shape, max_len, seed=0, unit_gains=False, head=True):
    from paper_2602_16760_amd.engine import Engine
    hw = synth.head_weights(shape, seed, unit_gains) if head else None
    return Engine(shape, max_len, lambda l: synth.layer_weights(shape, l, seed, unit_gains), hw)


def prefill_both(shape, eng, okv, L, seed=0):
    """Cache rows 0..L-1 of every layer ~ N(0,1) on both sides; sets both lengths to L."""
    from paper_2602_16760_amd import binding as B
    for l in range(shape.n_layers):
        k, v = synth.kv_fill(shape, l, L, seed)
        okv.fill(l, k, v)
        eng.fill_kv(l, k, v)
    okv.L = L
    B.la_kv_set_len(eng.kv, L)


def row_rel_err(got, want):
    """Per row: max |got - want| / max |want| (the parity metric for hidden states)."""
    got = np.asarray(got, dtype=np.float64)
    want = np.asarray(want, dtype=np.float64)
    return np.max(np.abs(got - want), axis=-1) / np.max(np.abs(want), axis=-1)
