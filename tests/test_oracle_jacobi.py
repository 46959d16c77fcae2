"""Pins of the Jacobi decoding oracle (oracle/jacobi.py; Section 4.2): its fixed point is the
greedy continuation, on fake models with known answers and on the float64 tiny decoder."""
import numpy as np
import pytest

import synth
from oracle import jacobi as jc
from oracle import rtt
from oracle import transformer as tf


def _pseudo_sequences(prefix, tok, pos, vis):
    out = []
    for i in range(len(tok)):
        rows = sorted([j for j in range(len(tok)) if vis[i] >> j & 1], key=lambda j: pos[j])
        out.append(list(prefix) + [tok[j] for j in rows])
    return out


def _run_fake(f, prompt, n_new, k, Bp=None):
    """Drive the controller with a 'model' whose next token is f(everything the row sees)."""
    st = jc.JacobiState(prompt, k, Bp)
    committed = list(prompt[:-1])
    iters, greedy = [], list(prompt)
    while len(st.emitted) < n_new:
        tok, pos, vis = st.block()
        assert st.t == len(committed) and pos[:k] == list(range(st.t, st.t + k))
        ids = [f(s) for s in _pseudo_sequences(committed, tok, pos, vis)]
        # after j iterations on a block the first j guesses are the greedy tokens (and stay)
        j = st.it
        c0 = st.c0
        out = st.step(ids, n_new - len(st.emitted))
        if out:
            iters.append(st.last_iterations)
            committed += [c0] + out[:-1]
        else:
            want = list(prompt) + st.emitted
            for _ in range(j + 1):
                want.append(f(want))
            assert st.y[:j + 1] == want[len(prompt) + len(st.emitted):]
    return st, iters


def _sequential(f, prompt, n_new):
    seq = list(prompt)
    for _ in range(n_new):
        seq.append(f(seq))
    return seq[len(prompt):]


@pytest.mark.parametrize("k", [1, 2, 5, 8])
def test_fixed_point_is_the_greedy_stream_on_a_context_dependent_fake_model(k):
    V = 23
    f = lambda s: (s[-1] * 7 + (s[-2] if len(s) > 1 else 0) * 3 + (len(s) % 5 == 0)) % V
    prompt = [int(x) for x in synth.uniform_prompt(V, 12, k)]
    st, iters = _run_fake(f, prompt, 41, k)
    assert st.emitted == _sequential(f, prompt, 41)
    assert all(1 <= i <= k for i in iters) and st.iterations == sum(iters)
    assert st.blocks == len(iters) == -(-41 // k)


def test_successor_model_needs_k_iterations_and_constant_model_two():
    k = 6
    succ = lambda s: (s[-1] + 1) % 50             # each iteration fixes exactly one more position
    st, iters = _run_fake(succ, [3, 4, 5], 24, k)
    assert st.emitted == [(6 + i) % 50 for i in range(24)] and iters == [k] * 4
    const = lambda s: 7                            # the second pass returns what the first one gave
    st, iters = _run_fake(const, [3, 4, 5], 24, k)
    assert st.emitted == [7] * 24 and iters[0] == 2 and iters[1:] == [1] * 3   # later blocks start from c0 = 7
    # Section 4.2's relation on these runs: tokens per second at a 100 ms round trip
    assert rtt.jacobi_tok_s(k, 2, 100.0) == 30.0 and rtt.jacobi_tok_s(k, k, 100.0) == 10.0


def test_budget_truncation_and_pad_rows():
    succ = lambda s: (s[-1] + 1) % 50
    st, iters = _run_fake(succ, [1, 2], 7, 4, Bp=6)
    assert st.emitted == [3, 4, 5, 6, 7, 8, 9] and st.t == 1 + 7
    tok, pos, vis = jc.JacobiState([1, 2], 4, Bp=6).block()
    assert len(tok) == 6 and vis[4:] == [1 << 4, 1 << 5] and vis[:4] == [1, 3, 7, 15]


def _tiny(seed):
    sh = synth.SHAPES["tiny_f32"]
    return tf.Model(sh, lambda l: synth.layer_weights(sh, l, seed), synth.head_weights(sh, seed))


@pytest.mark.parametrize("k,seed", [(4, 0), (7, 1)])
def test_tiny_decoder_jacobi_equals_sequential_and_cache_equals_sequential_cache(k, seed):
    model = _tiny(seed)
    prompt = synth.uniform_prompt(model.shape.vocab, 16, seed)
    seq, _, kv_seq = tf.greedy_sequential(model, prompt, 20, return_logits=True)
    out, st, kv = jc.greedy_jacobi(model, prompt, 20, k, Bp=8)
    assert np.array_equal(out, seq)
    assert st.iterations <= 20 + st.blocks and all(x >= 0 for x in out)
    n = min(kv.L, kv_seq.L)
    assert kv.L == len(prompt) - 1 + 20
    assert np.allclose(kv.K[:, :n], kv_seq.K[:, :n], atol=1e-11)
    assert np.allclose(kv.V[:, :n], kv_seq.V[:, :n], atol=1e-11)
