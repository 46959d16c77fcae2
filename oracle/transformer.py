"""Float64 Mistral-family decoder stack (test oracle; see package docstring).

The paper names the model family only (Section 3.1: RMS norm + LM head,
grouped-query attention with 8 KV heads against 32 query heads; Section 8:
MistralForCausalLM).  The layer arithmetic is that family's published
definition:

    h  = x * rsqrt(mean(x^2) + eps) * g_attn
    q, k, v = h Wq, h Wk, h Wv;   q, k rotated by RoPE at the row's position
    a_h = softmax(q_h . k_{kv(h)} / sqrt(dh)) v_{kv(h)},  kv(h) = h // (Hq/Hkv)
    x  = x + concat(a) Wo
    x  = x + (silu(h2 Wg) * (h2 Wu)) Wd,   h2 = rmsnorm(x, g_mlp)
    logits = rmsnorm(x, g_final) U

RoPE uses the half-split pairing: element i is paired with element i + dh/2
and the pair is rotated by the angle pos * theta^(-2i/dh).
Keys are cached after rotation.  Every weight matrix is row-major [in, out].
"""
from __future__ import annotations

import numpy as np

F64 = np.float64


def widen(a: np.ndarray) -> np.ndarray:
    """Storage array (float32, or bfloat16 bit patterns as uint16) -> float64."""
    if a.dtype == np.uint16:
        return (a.astype(np.uint32) << np.uint32(16)).view(np.float32).astype(F64)
    return a.astype(F64)


class Model:
    """Holds the stored weights; widens one layer at a time on demand.

    `layer_source(l)` returns the dict of stored arrays for layer l (see
    synth.layer_weights).  `head` holds embed / g_final / unembed as stored.
    With cache=True the widened layers are kept (small models only).
    """

    def __init__(self, shape, layer_source, head=None, cache=True):
        self.shape = shape
        self._src = layer_source
        self._cache = {} if cache else None
        self.head = {k: widen(v) for k, v in (head or {}).items()}

    def layer(self, l: int) -> dict:
        if self._cache is not None and l in self._cache:
            return self._cache[l]
        w = {k: widen(v) for k, v in self._src(l).items()}
        if self._cache is not None:
            self._cache[l] = w
        return w


class KVCache:
    """Per-layer K, V [max_len, Hkv, dh] float64 and the committed length L.

    Rows 0..L-1 are committed (row index = token position).  A block forward
    writes its rows at L..L+B-1; they stay scratch until committed.
    """

    def __init__(self, shape, max_len: int, n_layers: int | None = None):
        nl = shape.n_layers if n_layers is None else n_layers
        self.K = np.zeros((nl, max_len, shape.n_kv_heads, shape.head_dim), F64)
        self.V = np.zeros_like(self.K)
        self.L = 0

    def fill(self, layer: int, k: np.ndarray, v: np.ndarray):
        n = k.shape[0]
        self.K[layer, :n] = widen(k)
        self.V[layer, :n] = widen(v)

    def move_rows(self, moves):
        """Apply (src_row, dst_row) copies to every layer, in list order."""
        for src, dst in moves:
            if src != dst:
                self.K[:, dst] = self.K[:, src]
                self.V[:, dst] = self.V[:, src]


def rmsnorm(x, g, eps):
    return x / np.sqrt(np.mean(x * x, axis=-1, keepdims=True) + eps) * g


def rope(u, pos, theta):
    """u [B, H, dh], pos [B] -> rotated copy (half-split pairing)."""
    dh = u.shape[-1]
    half = dh // 2
    inv = theta ** (-2.0 * np.arange(half, dtype=F64) / dh)
    phi = np.asarray(pos, dtype=F64)[:, None] * inv[None, :]
    c = np.cos(phi)[:, None, :]
    s = np.sin(phi)[:, None, :]
    a, b = u[..., :half], u[..., half:]
    return np.concatenate([a * c - b * s, b * c + a * s], axis=-1)


def silu(z):
    return z / (1.0 + np.exp(-z))


def softmax(s):
    e = np.exp(s - np.max(s))
    return e / np.sum(e)


def visible_block_rows(vis_bits: int, n_rows: int):
    return [j for j in range(n_rows) if (int(vis_bits) >> j) & 1]


def forward_block(model: Model, kv: KVCache, x, pos, vis, layer_begin=0, layer_end=None,
                  kv_layer_offset=0, progress=None):
    """Push a block of B rows through layers [layer_begin, layer_end).

    x [B, d] residual stream (float64), pos [B] positions, vis [B] integers:
    bit j of vis[b] set <=> row b attends to block row j.  Every row also
    attends to all committed cache rows (< kv.L).  The block's K, V are written
    to cache rows L..L+B-1 of each layer (Section 3.3: the cloud keeps the
    cache; Section 4.4: explicit masks for multi-token steps).
    kv_layer_offset: cache layer index = model layer index - kv_layer_offset.
    Returns the new residual stream [B, d].
    """
    sh = model.shape
    Hq, Hkv, dh = sh.n_q_heads, sh.n_kv_heads, sh.head_dim
    g = Hq // Hkv
    layer_end = sh.n_layers if layer_end is None else layer_end
    x = np.array(x, dtype=F64)
    B = x.shape[0]
    L = kv.L
    scale = 1.0 / np.sqrt(dh)
    for l in range(layer_begin, layer_end):
        w = model.layer(l)
        cl = l - kv_layer_offset
        h = rmsnorm(x, w["g_attn"], sh.rms_eps)
        q = rope((h @ w["wq"]).reshape(B, Hq, dh), pos, sh.rope_theta)
        k = rope((h @ w["wk"]).reshape(B, Hkv, dh), pos, sh.rope_theta)
        v = (h @ w["wv"]).reshape(B, Hkv, dh)
        kv.K[cl, L:L + B] = k
        kv.V[cl, L:L + B] = v
        a = np.zeros((B, Hq, dh), F64)
        for b in range(B):
            rows = visible_block_rows(vis[b], B)
            if L == 0 and not rows:
                raise ValueError(f"row {b} sees nothing")
            Kb = np.concatenate([kv.K[cl, :L], kv.K[cl, [L + j for j in rows]]], axis=0)
            Vb = np.concatenate([kv.V[cl, :L], kv.V[cl, [L + j for j in rows]]], axis=0)
            for hq in range(Hq):
                p = softmax((Kb[:, hq // g, :] @ q[b, hq]) * scale)
                a[b, hq] = p @ Vb[:, hq // g, :]
        x = x + a.reshape(B, Hq * dh) @ w["wo"]
        h2 = rmsnorm(x, w["g_mlp"], sh.rms_eps)
        x = x + (silu(h2 @ w["wgate"]) * (h2 @ w["wup"])) @ w["wdown"]
        if progress is not None:
            progress(l)
    return x


def logits_of(model: Model, x):
    sh = model.shape
    return rmsnorm(np.asarray(x, F64), model.head["g_final"], sh.rms_eps) @ model.head["unembed"]


def argmax_ids(logits):
    """Greedy choice per row; ties go to the lowest index."""
    return np.argmax(logits, axis=-1).astype(np.int64)


def top2_margin(logits):
    """Per row: (top-1 value, top-2 value) -- the margin is their difference."""
    part = np.partition(logits, -2, axis=-1)
    return part[..., -1], part[..., -2]


def embed(model: Model, tokens):
    return model.head["embed"][np.asarray(tokens, dtype=np.int64)]


def causal_forward(model: Model, tokens):
    """Dense full-sequence causal pass: the textbook definition of the model.

    tokens [T] -> (final residual stream [T, d], logits [T, V]).  Position t
    attends to positions 0..t.  No cache, no blocks: every layer works on the
    whole [T, T] score matrix.
    """
    sh = model.shape
    Hq, Hkv, dh = sh.n_q_heads, sh.n_kv_heads, sh.head_dim
    g = Hq // Hkv
    T = len(tokens)
    pos = np.arange(T)
    x = embed(model, tokens)
    allowed = np.tril(np.ones((T, T), dtype=bool))
    for l in range(sh.n_layers):
        w = model.layer(l)
        h = rmsnorm(x, w["g_attn"], sh.rms_eps)
        q = rope((h @ w["wq"]).reshape(T, Hq, dh), pos, sh.rope_theta)
        k = rope((h @ w["wk"]).reshape(T, Hkv, dh), pos, sh.rope_theta)
        v = (h @ w["wv"]).reshape(T, Hkv, dh)
        a = np.zeros((T, Hq, dh), F64)
        for hq in range(Hq):
            s = (q[:, hq, :] @ k[:, hq // g, :].T) / np.sqrt(dh)
            s = np.where(allowed, s, -np.inf)
            s = s - s.max(axis=1, keepdims=True)
            p = np.exp(s)
            p = p / p.sum(axis=1, keepdims=True)
            a[:, hq, :] = p @ v[:, hq // g, :]
        x = x + a.reshape(T, Hq * dh) @ w["wo"]
        h2 = rmsnorm(x, w["g_mlp"], sh.rms_eps)
        x = x + (silu(h2 @ w["wgate"]) * (h2 @ w["wup"])) @ w["wdown"]
    return x, logits_of(model, x)


def prefill(model: Model, kv: KVCache, tokens, chunk=64):
    """Fill cache rows kv.L.. with the given tokens (causal inside each chunk)."""
    tokens = np.asarray(tokens)
    last = None
    for s in range(0, len(tokens), chunk):
        blk = tokens[s:s + chunk]
        n = len(blk)
        pos = kv.L + np.arange(n)
        vis = [(1 << (i + 1)) - 1 for i in range(n)]
        last = forward_block(model, kv, embed(model, blk), pos, vis)
        kv.L += n
    return last


def greedy_sequential(model: Model, prompt, n_new, kv: KVCache | None = None, return_logits=False):
    """The sequential baseline (Section 4.1): one token per forward pass.

    Returns the n_new generated tokens.  The cache ends up holding
    prompt + generated[:-1].
    """
    prompt = np.asarray(prompt)
    if kv is None:
        kv = KVCache(model.shape, len(prompt) + n_new + 1)
    prefill(model, kv, prompt[:-1])
    cur = int(prompt[-1])
    out, all_logits = [], []
    for _ in range(n_new):
        x = forward_block(model, kv, embed(model, [cur]), [kv.L], [1])
        lg = logits_of(model, x)
        kv.L += 1
        cur = int(argmax_ids(lg)[0])
        out.append(cur)
        if return_logits:
            all_logits.append(lg[0])
    if return_logits:
        return np.asarray(out, dtype=np.int64), np.stack(all_logits), kv
    return np.asarray(out, dtype=np.int64)
