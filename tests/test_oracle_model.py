"""Pins for oracle/transformer.py (CPU only).

Each test checks the oracle against something other than itself: closed forms,
values worked with the math module (tests/golden/closed_forms.txt), an
independent torch float64 implementation built on library routines, and the
dense causal pass as the definition of the cached / blocked passes.
"""
import math
import os

import numpy as np
import pytest
import torch

import synth
from oracle import transformer as tf

GOLD = os.path.join(os.path.dirname(__file__), "golden")


def tiny_model(name="tiny_f32", seed=0, **over):
    sh = synth.SHAPES[name]
    if over:
        from dataclasses import replace
        sh = replace(sh, **over)
    head = synth.head_weights(sh, seed)
    return tf.Model(sh, lambda l: synth.layer_weights(sh, l, seed), head)


def golden_lines(fname, tag):
    out = []
    for ln in open(os.path.join(GOLD, fname)):
        if ln.startswith(tag + " "):
            out.append(ln.split()[1:])
    return out


# ---------------------------------------------------------------- closed forms
def test_silu_golden():
    for z, want in golden_lines("closed_forms.txt", "silu"):
        assert abs(tf.silu(np.float64(z)) - float(want)) < 1e-15


def test_rope_golden_and_invariants():
    u = np.array([[[1.0, 2.0, 3.0, 4.0]]])
    got = tf.rope(u, [3], 10000.0)[0, 0]
    for i, want in golden_lines("closed_forms.txt", "rope"):
        assert abs(got[int(i)] - float(want)) < 1e-14
    rng = np.random.default_rng(1)
    q = rng.standard_normal((5, 3, 64))
    k = rng.standard_normal((5, 3, 64))
    pos = np.array([0, 7, 100, 3000, 4095])
    rq = tf.rope(q, pos, 1e6)
    # rotation keeps norms; position 0 is the identity
    assert np.allclose(np.linalg.norm(rq, axis=-1), np.linalg.norm(q, axis=-1), rtol=1e-13)
    assert np.array_equal(rq[0], q[0])
    # scores depend on position differences only
    s0 = np.einsum("bhd,chd->bch", rq, tf.rope(k, pos, 1e6))
    s1 = np.einsum("bhd,chd->bch", tf.rope(q, pos + 17, 1e6), tf.rope(k, pos + 17, 1e6))
    assert np.allclose(s0, s1, atol=1e-9)


def test_rmsnorm_unit_rms_and_gain():
    rng = np.random.default_rng(2)
    x = rng.standard_normal((4, 256)) * 3.0
    y = tf.rmsnorm(x, np.ones(256), 0.0)
    assert np.allclose(np.sqrt(np.mean(y * y, axis=-1)), 1.0, rtol=1e-13)
    g = rng.random(256) + 0.5
    assert np.allclose(tf.rmsnorm(x, g, 0.0), y * g)
    # eps enters under the square root, next to the mean square
    one = tf.rmsnorm(np.full((1, 8), 2.0), np.ones(8), 5.0)
    assert np.allclose(one, 2.0 / math.sqrt(4.0 + 5.0))


def test_softmax_rows():
    s = np.array([1.0, 2.0, 3.0])
    p = tf.softmax(s)
    assert abs(p.sum() - 1) < 1e-15
    assert np.allclose(p, np.exp(s) / np.exp(s).sum())
    assert np.allclose(tf.softmax(s + 1000.0), p)


def test_argmax_ties_lowest_and_bruteforce():
    rng = np.random.default_rng(3)
    lg = rng.standard_normal((6, 50))
    lg[2, 7] = lg[2, 31] = 99.0
    ids = tf.argmax_ids(lg)
    assert ids[2] == 7
    for r in range(6):
        best = 0
        for v in range(50):
            if lg[r, v] > lg[r, best]:
                best = v
        assert ids[r] == best
    t1, t2 = tf.top2_margin(lg)
    assert t1[2] == 99.0 and t2[2] == 99.0
    srt = np.sort(lg, axis=-1)
    assert np.array_equal(t1, srt[:, -1]) and np.array_equal(t2, srt[:, -2])


# ------------------------------------------------- attention special cases
def _probe_model(sh, wq_zero=False, seed=5):
    """Layer with Wo = I and a zero MLP, so that out - x is the attention output."""
    assert sh.q_dim == sh.d_model
    w = synth.layer_weights(sh, 0, seed)
    w["wo"] = np.eye(sh.d_model, dtype=np.float32)
    w["wdown"] = np.zeros_like(w["wdown"])
    if wq_zero:
        w["wq"] = np.zeros_like(w["wq"])
    return tf.Model(sh.with_layers(1), lambda l: w), w


def test_single_row_empty_cache_attention_is_v():
    sh = synth.SHAPES["tiny_f32"]
    model, w = _probe_model(sh)
    x = synth.hidden_block(sh, 1, 3).astype(np.float64)
    kv = tf.KVCache(sh, 4, 1)
    out = tf.forward_block(model, kv, x, [5], [1])
    v = (tf.rmsnorm(x, w["g_attn"].astype(np.float64), sh.rms_eps) @ w["wv"].astype(np.float64))
    v = v.reshape(sh.n_kv_heads, sh.head_dim)
    g = sh.n_q_heads // sh.n_kv_heads
    want = np.concatenate([v[h // g] for h in range(sh.n_q_heads)])
    assert np.allclose(out[0] - x[0], want, atol=1e-13)


def test_uniform_scores_give_mean_of_visible_values():
    sh = synth.SHAPES["tiny_f32"]
    model, w = _probe_model(sh, wq_zero=True)
    kv = tf.KVCache(sh, 16, 1)
    kf, vf = synth.kv_fill(sh, 0, 3, 1)
    kv.fill(0, kf, vf)
    kv.L = 3
    x = synth.hidden_block(sh, 4, 4).astype(np.float64)
    vis = [0b0001, 0b0011, 0b0101, 0b1011]
    out = tf.forward_block(model, kv, x, [3, 4, 4, 5], vis)
    V = kv.V[0]
    g = sh.n_q_heads // sh.n_kv_heads
    for b in range(4):
        rows = [0, 1, 2] + [3 + j for j in range(4) if vis[b] >> j & 1]
        m = V[rows].mean(axis=0)
        want = np.concatenate([m[h // g] for h in range(sh.n_q_heads)])
        assert np.allclose(out[b] - x[b], want, atol=1e-13)


def test_gqa_equals_mha_with_repeated_kv_heads():
    sh = synth.SHAPES["tiny_f32"]
    from dataclasses import replace
    w = synth.layer_weights(sh, 0, 7)
    g = sh.n_q_heads // sh.n_kv_heads
    dh = sh.head_dim

    def rep(m):  # [d, Hkv*dh] -> [d, Hq*dh]: kv head j serves q heads j*g .. j*g+g-1
        m = m.reshape(sh.d_model, sh.n_kv_heads, dh)
        return np.repeat(m, g, axis=1).reshape(sh.d_model, sh.n_q_heads * dh)

    w2 = dict(w, wk=rep(w["wk"]), wv=rep(w["wv"]))
    sh2 = replace(sh, n_kv_heads=sh.n_q_heads)
    head = synth.head_weights(sh, 7)
    toks = synth.uniform_prompt(sh.vocab, 9, 7)
    a = tf.causal_forward(tf.Model(sh.with_layers(1), lambda l: w, head), toks)[0]
    b = tf.causal_forward(tf.Model(sh2.with_layers(1), lambda l: w2, head), toks)[0]
    assert np.allclose(a, b, atol=1e-12)


# ------------------------------------- independent implementation on library ops
def _torch_causal(sh, layers, head, toks):
    """Same model written on torch float64 library routines: F.rms_norm,
    complex-number RoPE, F.scaled_dot_product_attention(is_causal=True),
    F.silu, F.embedding.  Shares nothing with the oracle."""
    F = torch.nn.functional
    T = len(toks)
    t64 = lambda a: torch.from_numpy(np.asarray(a, dtype=np.float64))
    x = F.embedding(torch.from_numpy(np.asarray(toks, dtype=np.int64)), t64(head["embed"]))
    half = sh.head_dim // 2
    freqs = 1.0 / (sh.rope_theta ** (torch.arange(0, sh.head_dim, 2, dtype=torch.float64) / sh.head_dim))
    ang = torch.outer(torch.arange(T, dtype=torch.float64), freqs)
    rot = torch.polar(torch.ones_like(ang), ang)  # e^{i pos w_i}, [T, half]

    def rope(u):  # [T, H, dh]; pair (i, i+half) is one complex number
        z = torch.complex(u[..., :half], u[..., half:]) * rot[:, None, :]
        return torch.cat([z.real, z.imag], dim=-1)

    for w in layers:
        h = F.rms_norm(x, (sh.d_model,), t64(w["g_attn"]), sh.rms_eps)
        q = rope(F.linear(h, t64(w["wq"]).T).view(T, sh.n_q_heads, sh.head_dim))
        k = rope(F.linear(h, t64(w["wk"]).T).view(T, sh.n_kv_heads, sh.head_dim))
        v = F.linear(h, t64(w["wv"]).T).view(T, sh.n_kv_heads, sh.head_dim)
        g = sh.n_q_heads // sh.n_kv_heads
        k = k.repeat_interleave(g, dim=1)
        v = v.repeat_interleave(g, dim=1)
        a = F.scaled_dot_product_attention(q.transpose(0, 1)[None], k.transpose(0, 1)[None],
                                           v.transpose(0, 1)[None], is_causal=True)[0]
        x = x + F.linear(a.transpose(0, 1).reshape(T, sh.q_dim), t64(w["wo"]).T)
        h2 = F.rms_norm(x, (sh.d_model,), t64(w["g_mlp"]), sh.rms_eps)
        x = x + F.linear(F.silu(F.linear(h2, t64(w["wgate"]).T)) * F.linear(h2, t64(w["wup"]).T),
                         t64(w["wdown"]).T)
    lg = F.linear(F.rms_norm(x, (sh.d_model,), t64(head["g_final"]), sh.rms_eps), t64(head["unembed"]).T)
    return x.numpy(), lg.numpy()


@pytest.mark.parametrize("name", ["tiny_f32", "small64_bf16"])
def test_causal_forward_matches_torch_library_model(name):
    sh = synth.SHAPES[name].with_layers(2)
    layers = [synth.layer_weights(sh, l, 11) for l in range(2)]
    head = synth.head_weights(sh, 11)
    wide = lambda d: {k: tf.widen(v) for k, v in d.items()}
    toks = synth.uniform_prompt(sh.vocab, 13, 11)
    x0, lg0 = tf.causal_forward(tf.Model(sh, lambda l: layers[l], head), toks)
    x1, lg1 = _torch_causal(sh, [wide(w) for w in layers], wide(head), toks)
    assert np.allclose(x0, x1, atol=1e-11, rtol=1e-11)
    assert np.allclose(lg0, lg1, atol=1e-11, rtol=1e-11)


# --------------------------------- cached / blocked passes against the definition
def test_sequential_cache_decode_equals_dense_recompute():
    model = tiny_model()
    prompt = synth.uniform_prompt(model.shape.vocab, 12, 1)
    toks, lgs, kv = tf.greedy_sequential(model, prompt, 6, return_logits=True)
    stream = np.concatenate([prompt, toks])
    xs, dense = tf.causal_forward(model, stream[:-1])
    assert np.allclose(dense[len(prompt) - 1:], lgs, atol=1e-11)
    assert np.array_equal(np.argmax(dense[len(prompt) - 1:], axis=-1), toks)
    # brute force: regenerate each token from a dense pass on its whole prefix
    cur = list(prompt)
    for t in toks[:3]:
        nxt = int(np.argmax(tf.causal_forward(model, cur)[1][-1]))
        assert nxt == t
        cur.append(nxt)


def test_printed_causal_mask_special_case_and_relative_mask_failure():
    """Section 4.4: with k speculative rows after a committed cache, row i must see
    cache[:committed] and block rows <= i.  That reproduces the dense causal pass;
    a mask laid out relative to the block alone (as if there were no cache) does not."""
    from oracle.lookahead import causal_block
    model = tiny_model()
    sh = model.shape
    toks = synth.uniform_prompt(sh.vocab, 15, 2)
    committed, k = 9, 6
    kv = tf.KVCache(sh, 32)
    tf.prefill(model, kv, toks[:committed])
    pos, vis = causal_block(committed, k)
    x = tf.forward_block(model, kv, tf.embed(model, toks[committed:]), pos, vis)
    dense = tf.causal_forward(model, toks)[0]
    assert np.allclose(x, dense[committed:], atol=1e-11)
    # the failure the paper warns of: a mask built relative to the block alone.  With a
    # non-empty cache, is_causal-style masking aligns the triangle to the top-left corner
    # of the k x kv_len score matrix, so speculative row i sees kv entries 0..i only.
    # Emulate it by treating the whole kv axis as one block over an empty cache.
    kv_len = committed + k
    kvr = tf.KVCache(sh, 32)
    xr = tf.forward_block(model, kvr, tf.embed(model, toks), np.arange(kv_len),
                          [(1 << (max(i - committed, 0) + 1)) - 1 if i >= committed else (1 << (i + 1)) - 1
                           for i in range(kv_len)])
    assert not np.allclose(xr[committed:], dense[committed:], atol=1e-3)
    # and the other obvious wrong masks: self only, or everything in the block
    for bad in ([1 << i for i in range(k)], [(1 << k) - 1] * k):
        kvb = tf.KVCache(sh, 32)
        tf.prefill(model, kvb, toks[:committed])
        xb = tf.forward_block(model, kvb, tf.embed(model, toks[committed:]), pos, bad)
        assert not np.allclose(xb[1:-1], dense[committed + 1:-1], atol=1e-3)


def test_block_rows_under_lookahead_mask_equal_their_pseudo_sequences():
    from oracle import lookahead as la
    model = tiny_model()
    sh = model.shape
    W, N, G = 3, 3, 2
    prompt = synth.uniform_prompt(sh.vocab, 10, 4)
    st = la.LookaheadState(prompt, W, N, G, Bp=16)
    # force two candidates so the verify rows are exercised
    st.cands = [(5, 6), (7, 8)]
    tok, pos, vis = st.block()
    kv = tf.KVCache(sh, 64)
    tf.prefill(model, kv, prompt[:-1])
    x = tf.forward_block(model, kv, tf.embed(model, tok), pos, vis)
    lg = tf.logits_of(model, x)
    for i in range(16):
        rows = sorted([j for j in range(16) if vis[i] >> j & 1], key=lambda j: pos[j])
        assert [pos[j] for j in rows] == list(range(st.t, st.t + len(rows)))
        assert rows[-1] == i
        seq = list(prompt[:-1]) + [tok[j] for j in rows]
        xd, lgd = tf.causal_forward(model, seq)
        assert np.allclose(x[i], xd[-1], atol=1e-11)
        assert np.allclose(lg[i], lgd[-1], atol=1e-11)
