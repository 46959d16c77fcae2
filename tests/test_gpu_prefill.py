"""The prompt pass (la_prefill): the large-M path (one matrix product per weight matrix and prompt
chunk) and the chunked path through the block kernel, against the oracle's prefill and each other."""
import numpy as np
import pytest

import synth
from gpu_util import gpu_engine, oracle_model, row_rel_err
from oracle import transformer as otf

pytestmark = pytest.mark.gpu
TOL = {"bf16": 2e-2, "f16": 2e-3}   # (cache rows: one storage rounding, 2^-9 resp. 2^-12 of the largest element, on top of the hidden-state error)


def _cache_rows(eng, shape, n):
    out = []
    for l in range(shape.n_layers):
        k, v = eng.read_kv(l, 0, n)
        if shape.dtype == "bf16":
            k, v = synth.bf16_to_f32(k), synth.bf16_to_f32(v)
        out.append((np.asarray(k, dtype=np.float64), np.asarray(v, dtype=np.float64)))
    return out


@pytest.mark.parametrize("name,n_tok", [("small_bf16", 300), ("small64_bf16", 129), ("small_f16", 200), ("small_bf16", 1100)])
def test_large_prompt_pass_matches_oracle_and_the_chunked_pass(name, n_tok):
    import torch
    from paper_2602_16760_amd import binding as B
    shape = synth.SHAPES[name]
    toks = synth.uniform_prompt(shape.vocab, n_tok, 5)
    om = oracle_model(shape, seed=6)
    okv = otf.KVCache(shape, n_tok + 64)
    otf.prefill(om, okv, toks)
    big = gpu_engine(shape, n_tok + 64, seed=6)
    small = gpu_engine(shape, n_tok + 64, seed=6)
    try:
        td = B.to_device(np.asarray(toks, dtype=np.int32))
        B.la_prefill(big.model, big.kv, td, 0)                       # 128 tokens or more: the large-M pass
        assert B.la_kv_get_len(big.kv) == n_tok
        for s in range(0, n_tok, 100):                               # pieces below 128 tokens: the block kernel
            B.la_prefill(small.model, small.kv, td[s:s + 100].contiguous(), s)
        assert B.la_kv_get_len(small.kv) == n_tok
        torch.cuda.synchronize()
        tol = TOL[shape.dtype]
        worst = 0.0
        for l, ((kb, vb), (ks, vs)) in enumerate(zip(_cache_rows(big, shape, n_tok), _cache_rows(small, shape, n_tok))):
            ko, vo = okv.K[l, :n_tok], okv.V[l, :n_tok]
            for got in (kb, ks):
                e = np.max(np.abs(got - ko)) / np.max(np.abs(ko))
                worst = max(worst, e)
                assert e <= tol, f"layer {l} K: {e:.3e}"
            for got in (vb, vs):
                e = np.max(np.abs(got - vo)) / np.max(np.abs(vo))
                worst = max(worst, e)
                assert e <= tol, f"layer {l} V: {e:.3e}"
            assert np.max(np.abs(kb - ks)) <= 2 * tol * np.max(np.abs(ko)) and np.max(np.abs(vb - vs)) <= 2 * tol * np.max(np.abs(vo))
        print(f"{name}, {n_tok} tokens: worst cache error against the oracle {worst:.3e}")
        # a decode block on top of either cache: same hidden states within the bar of the oracle
        x = synth.hidden_block(shape, 8, 3)
        pos = [n_tok + i for i in range(8)]
        vis = [(1 << (i + 1)) - 1 for i in range(8)]
        okv.L = n_tok
        want = otf.forward_block(om, okv, x, pos, vis)
        assert row_rel_err(big.forward(x, pos, vis), want).max() <= tol
        assert row_rel_err(small.forward(x, pos, vis), want).max() <= tol
    finally:
        big.close()
        small.close()


def test_generation_after_a_large_prompt_pass_equals_sequential():
    """The closed-form successor model: a 200-token prompt through the large-M pass, then lookahead
    and sequential generation give the orbit (the prompt's cache rows are what the steps attend to)."""
    from paper_2602_16760_amd.engine import Engine
    from test_gpu_parity import _orbit_model
    shape = synth.SHAPES["small_bf16"]
    period = 5
    perm, layer, head = _orbit_model(shape, period, 4)
    prompt = [3 * period + 2]
    for _ in range(199):
        prompt.append(int(perm[prompt[-1]]))
    prompt = np.asarray(prompt, dtype=np.int32)
    expect, cur = [], int(prompt[-1])
    for _ in range(40):
        cur = int(perm[cur])
        expect.append(cur)
    eng = Engine(shape, 512, layer, head)
    try:
        la, st = eng.generate(prompt, 40, 5, 4, 5, Bp=32)
        seq, _ = eng.generate(prompt, 40, 0, 1, 0)
        assert list(la) == expect and list(seq) == expect
        assert st["matched_steps"] > 0 and st["steps"] < 40
    finally:
        eng.close()
