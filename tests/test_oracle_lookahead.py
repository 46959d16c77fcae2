"""Pins for oracle/lookahead.py and the end-to-end invariant (CPU only).

The paper's Section 6.5 invariant is the strongest pin: greedy lookahead output
is token-identical to sequential greedy output.  It is checked on the float64
transformer (BASELINE config 1 and variants) and, for the integer logic alone,
on synthetic "models" that are pure functions of the prefix, where the expected
stream is known in closed form.
"""
import os

import numpy as np
import pytest

import synth
from oracle import lookahead as la
from oracle import transformer as tf

GOLD = os.path.join(os.path.dirname(__file__), "golden")


def test_block_layout_golden_w2_n3_g1():
    rows = [ln.split() for ln in open(os.path.join(GOLD, "la_layout_w2_n3_g1.txt")) if ln[0] != "#"]
    sym = {"c0": 100, "w00": 200, "w01": 201, "w10": 210, "w11": 211, "g1": 301, "g2": 302}
    t = 40
    tok, pos, vis = la.build_block(sym["c0"], t, [[200, 201], [210, 211]], [(301, 302)], 2, 3, 1)
    assert la.block_rows(2, 3, 1) == len(rows) == 7
    for r, s, dp, m in rows:
        r = int(r)
        assert tok[r] == sym[s] and pos[r] == t + int(dp) and vis[r] == int(m, 16)


def test_block_sizes_of_the_benchmark_configs():
    # BASELINE configs: W=4,N=3,G=4 -> 17; W=5,N=4,G=5 -> 31 (padded to 32); W=7,N=4,G=7 -> 43
    assert la.block_rows(4, 3, 4) == 17
    assert la.block_rows(5, 4, 5) == 31
    assert la.block_rows(7, 4, 7) == 43


def test_unused_and_pad_rows_see_only_themselves():
    tok, pos, vis = la.build_block(9, 5, [[1, 2], [3, 4]], [], 2, 3, 2, Bp=16)
    for i in range(5, 16):
        assert tok[i] == 9 and pos[i] == 5 and vis[i] == 1 << i


def test_pool_capacity_refresh_eviction_order():
    p = la.NgramPool(3, 2)
    p.insert(1, (10, 11))
    p.insert(1, (20, 21))
    assert p.lookup(1) == [(20, 21), (10, 11)]
    p.insert(1, (10, 11))                      # refresh, no duplicate
    assert p.lookup(1) == [(10, 11), (20, 21)]
    p.insert(1, (30, 31))                      # evicts the stalest: (20, 21)
    assert p.lookup(1) == [(30, 31), (10, 11)]
    assert p.lookup(2) == []
    q = la.NgramPool(3, 4)
    q.seed([1, 2, 3, 1, 2, 4, 1])
    # 3-grams starting at each position i <= P-3
    assert q.lookup(1) == [(2, 4), (2, 3)]
    assert q.lookup(2) == [(4, 1), (3, 1)]
    assert q.lookup(4) == []


def test_verify_match_lengths():
    W, N, G = 2, 4, 3
    v = lambda k, j: la.v_row(W, N, G, k, j)
    ids = [0] * la.block_rows(W, N, G)
    ids[0] = 7
    cands = [(7, 8, 9), (7, 5, 5), (6, 8, 9)]
    ids[v(0, 1)] = 8; ids[v(0, 2)] = 1          # cand 0 matches 7, 8 then fails -> m=2
    ids[v(1, 1)] = 5; ids[v(1, 2)] = 5          # cand 1 matches all three -> m=3
    ids[v(2, 1)] = 8; ids[v(2, 2)] = 9          # cand 2 fails on its first token -> m=0
    assert la.verify(ids, cands, W, N, G) == (1, 3)
    assert la.verify(ids, cands[:1], W, N, G) == (0, 2)
    assert la.verify(ids, [], W, N, G) == (0, 0)
    # ties go to the lowest k
    ids[v(0, 1)] = 5; ids[v(0, 2)] = 5
    assert la.verify(ids, [cands[1], cands[1]], W, N, G) == (0, 3)


# ---------------------------------------------- integer logic on synthetic models
def _pseudo_sequences(prefix, tok, pos, vis):
    out = []
    for i in range(len(tok)):
        rows = sorted([j for j in range(len(tok)) if vis[i] >> j & 1], key=lambda j: pos[j])
        out.append(list(prefix) + [tok[j] for j in rows])
    return out


def _run_fake(f, prompt, n_new, W, N, G, Bp=None, seed_pool=True):
    """Drive the controller with a 'model' whose next token is f(prefix)."""
    st = la.LookaheadState(prompt, W, N, G, Bp, seed_pool)
    committed = list(prompt[:-1])
    per_step = []
    while len(st.emitted) < n_new:
        tok, pos, vis = st.block()
        assert st.t == len(committed)
        ids = [f(s) for s in _pseudo_sequences(committed, tok, pos, vis)]
        c0 = st.c0
        out, moves = st.step(ids, n_new - len(st.emitted))
        # the moved rows must hold exactly the tokens that now sit at those positions
        assert all(tok[s] == ([c0] + out)[d] for s, d in moves)
        assert [d for _, d in moves] == list(range(1, len(out)))
        committed += [c0] + out[:-1]
        per_step.append(len(out))
    return st, per_step


def _sequential(f, prompt, n_new):
    seq = list(prompt)
    for _ in range(n_new):
        seq.append(f(seq))
    return seq[len(prompt):]


@pytest.mark.parametrize("W,N,G", [(4, 3, 4), (5, 4, 5), (1, 2, 1), (3, 2, 0), (2, 5, 3), (7, 4, 7)])
def test_fake_model_stream_identical_and_bounded(W, N, G):
    V = 23
    f = lambda s: (s[-1] * 7 + s[-2] * 3 + (len(s) % 5 == 0)) % V   # depends on length too: aperiodic-ish
    prompt = [int(x) for x in synth.uniform_prompt(V, 12, W + N + G)]
    st, per = _run_fake(f, prompt, 60, W, N, G)
    assert st.emitted == _sequential(f, prompt, 60)
    assert all(1 <= e <= N for e in per[:-1])      # Section 4.3: between 1 and n tokens per step
    assert sum(per) == 60


def test_periodic_text_reaches_n_tokens_per_step():
    V, W, N, G = 50, 4, 4, 4
    f = lambda s: (s[-1] + 1) % 10                  # 0,1,...,9,0,1,... : fully predictable from one token
    prompt = [3, 4, 5, 6, 7, 8, 9, 0, 1, 2, 3, 4, 5, 6, 7, 8, 9, 0, 1]
    st, per = _run_fake(f, prompt, 80, W, N, G)
    assert st.emitted == _sequential(f, prompt, 80)
    assert all(e == N for e in per[2:-1])           # pool seeded from the prompt already holds every 4-gram
    assert st.matched_steps >= len(per) - 2


def test_empty_pool_no_candidates_is_exactly_one_token_per_step():
    V = 1 << 20
    f = lambda s: (s[-1] * 1103515245 + 12345 + len(s)) % V     # never repeats within the run
    prompt = [5, 9, 11, 2]
    st, per = _run_fake(f, prompt, 40, 3, 3, 3, seed_pool=False)
    assert per == [1] * 40 and st.matched_steps == 0             # sequential rate: 1.00 tok/step
    st, per = _run_fake(f, prompt, 40, 3, 3, 0)                  # G = 0: never any candidate
    assert per == [1] * 40


def test_budget_truncation():
    f = lambda s: (s[-1] + 1) % 10
    prompt = [1, 2, 3, 4, 5, 6, 7, 8, 9, 0, 1, 2]
    st, per = _run_fake(f, prompt, 6, 4, 4, 4)
    assert st.emitted == _sequential(f, prompt, 6) and sum(per) == 6


# ----------------------------------------------------- the paper's invariant, fp64 model
def _tiny(seed=0):
    sh = synth.SHAPES["tiny_f32"]
    return tf.Model(sh, lambda l: synth.layer_weights(sh, l, seed), synth.head_weights(sh, seed))


def test_config1_lookahead_equals_sequential_and_cache_equals_sequential_cache():
    """BASELINE config 1: 2-layer tiny decoder, 32-token uniform prompt, W=4 N=3 G=4,
    32 generated tokens; lookahead == sequential, token for token (Section 6.5)."""
    model = _tiny(0)
    prompt = synth.uniform_prompt(model.shape.vocab, 32, 0)
    seq, _, kv_seq = tf.greedy_sequential(model, prompt, 32, return_logits=True)
    steps = []
    out, st, kv_la = la.greedy_lookahead(model, prompt, 32, 4, 3, 4, Bp=32, trace=lambda d: steps.append(d["L"]))
    assert np.array_equal(out, seq)
    assert len(out) == 32 and st.steps == len(steps) <= 32
    # after commit the committed cache rows are those of sequential decoding
    L = kv_la.L
    assert L == len(prompt) - 1 + 32
    n = min(L, kv_seq.L)
    assert np.allclose(kv_la.K[:, :n], kv_seq.K[:, :n], atol=1e-11)
    assert np.allclose(kv_la.V[:, :n], kv_seq.V[:, :n], atol=1e-11)


@pytest.mark.parametrize("W,N,G,seed", [(2, 2, 1, 1), (3, 4, 2, 2), (1, 3, 0, 3)])
def test_lookahead_equals_sequential_variants(W, N, G, seed):
    model = _tiny(seed)
    # a repetitive prompt so that candidates exist and some are accepted
    base = synth.uniform_prompt(model.shape.vocab, 6, seed)
    prompt = np.concatenate([base, base, base])
    seq = tf.greedy_sequential(model, prompt, 20)
    out, st, _ = la.greedy_lookahead(model, prompt, 20, W, N, G)
    assert np.array_equal(out, seq)
