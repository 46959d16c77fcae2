"""Integer logic of lookahead decoding (test oracle; see package docstring).

The paper (Section 4.3) describes lookahead decoding in two sentences: n-gram
candidates are collected from the trajectories of a Jacobi iteration, cached,
and verified in later steps so that several tokens can be committed per round
trip; Section 3.3 adds cache cropping, cache relocation and custom masks.  It
defines neither the window, the pool nor the mask.  The reading implemented
here (stated in full in the repository's design notes) uses three parameters:

    W  width of the lookahead window (columns of the Jacobi trajectory)
    N  n-gram size: a candidate is N-1 tokens following a key token
    G  maximum number of candidates verified per step

and a block of B = 1 + W(N-1) + G(N-1) rows per step:

    row 0                      the one real next-token row: token c0, position t
    la(r, c) = 1 + r W + c     window entry win[r][c], position t + 1 + c + r
    v(k, j)  = 1 + W(N-1) + k(N-1) + (j-1),  j = 1..N-1
                               candidate k's j-th token, position t + j

Visibility inside the block (all rows also see the whole committed cache):
    row 0    : itself
    la(r, c) : row 0, la(0, c') for c' <= c, la(r', c) for 1 <= r' <= r
    v(k, j)  : row 0, v(k, j') for j' <= j
    unused verify rows and pad rows: token c0, position t, see only themselves.
Each row's visible set has consecutive positions t, t+1, ..., so each row's
output is exactly the model's next-token prediction for its own pseudo-sequence.
"""
from __future__ import annotations

import numpy as np


def block_rows(W: int, N: int, G: int) -> int:
    return 1 + (W + G) * (N - 1)


def la_row(W, N, G, r, c):
    return 1 + r * W + c


def v_row(W, N, G, k, j):
    return 1 + W * (N - 1) + k * (N - 1) + (j - 1)


def build_block(c0, t, win, cands, W, N, G, Bp=None):
    """Rows of one step -> (tok[Bp], pos[Bp], vis[Bp]) as Python int lists.

    win[r][c] for r < N-1, c < W; cands: list of <= G tuples of N-1 tokens.
    """
    B = block_rows(W, N, G)
    Bp = B if Bp is None else Bp
    assert Bp >= B and Bp <= 64
    tok = [int(c0)] * Bp
    pos = [int(t)] * Bp
    vis = [1 << i for i in range(Bp)]
    vis[0] = 1
    for r in range(N - 1):
        for c in range(W):
            i = la_row(W, N, G, r, c)
            tok[i] = int(win[r][c])
            pos[i] = t + 1 + c + r
            m = 1
            for c2 in range(c + 1):
                m |= 1 << la_row(W, N, G, 0, c2)
            for r2 in range(1, r + 1):
                m |= 1 << la_row(W, N, G, r2, c)
            vis[i] = m
    for k, cand in enumerate(cands):
        assert k < G and len(cand) == N - 1
        for j in range(1, N):
            i = v_row(W, N, G, k, j)
            tok[i] = int(cand[j - 1])
            pos[i] = t + j
            m = 1
            for j2 in range(1, j + 1):
                m |= 1 << v_row(W, N, G, k, j2)
            vis[i] = m
    return tok, pos, vis


def causal_block(t, n):
    """The plain causal mask of Section 4.4: row i sees cache + block rows <= i."""
    return [t + i for i in range(n)], [(1 << (i + 1)) - 1 for i in range(n)]


class NgramPool:
    """Observed n-grams keyed by their first token (Section 4.3).

    Per key at most G distinct (N-1)-tuples.  Inserting a tuple that is already
    there refreshes its stamp; inserting into a full key evicts the entry with
    the smallest stamp.  lookup() returns the tuples most recent first.  Stamps
    come from one counter that advances on every insert.
    """

    def __init__(self, N: int, G: int):
        self.N, self.G = N, G
        self.table: dict[int, list] = {}
        self.stamp = 0

    def insert(self, key: int, tup):
        tup = tuple(int(x) for x in tup)
        assert len(tup) == self.N - 1
        self.stamp += 1
        if self.G == 0:
            return
        ent = self.table.setdefault(int(key), [])
        for e in ent:
            if e[0] == tup:
                e[1] = self.stamp
                return
        if len(ent) >= self.G:
            ent.remove(min(ent, key=lambda e: e[1]))
        ent.append([tup, self.stamp])

    def lookup(self, key: int):
        ent = self.table.get(int(key), [])
        return [e[0] for e in sorted(ent, key=lambda e: -e[1])]

    def seed(self, prompt):
        N = self.N
        for i in range(0, len(prompt) - N + 1):
            self.insert(prompt[i], prompt[i + 1:i + N])


def verify(ids, cands, W, N, G):
    """Longest candidate prefix confirmed by the model's own choices.

    ids[i] is the greedy token predicted at block row i.  Candidate k matches
    m_k tokens: g_1 must equal ids[0]; g_{j+1} must equal ids[v(k, j)].
    Returns (k*, m): the best candidate (ties -> lowest k) and its match length.
    """
    best_k, best_m = 0, 0
    for k, cand in enumerate(cands):
        m = 0
        if cand[0] == ids[0]:
            m = 1
            while m < N - 1 and cand[m] == ids[v_row(W, N, G, k, m)]:
                m += 1
        if m > best_m:
            best_k, best_m = k, m
    return best_k, best_m


class LookaheadState:
    """Controller state between steps; `step(ids)` is one accept phase."""

    def __init__(self, prompt, W, N, G, Bp=None, seed_pool=True):
        prompt = [int(x) for x in prompt]
        P = len(prompt)
        self.W, self.N, self.G = W, N, G
        self.Bp = block_rows(W, N, G) if Bp is None else Bp
        self.pool = NgramPool(N, G)
        if seed_pool:
            self.pool.seed(prompt)
        self.win = [[prompt[(r + c) % P] for c in range(W)] for r in range(N - 1)]
        self.t = P - 1          # position of c0 = committed cache length L
        self.c0 = prompt[-1]
        self.cands = self.pool.lookup(self.c0)[:G]
        self.steps = 0
        self.matched_steps = 0
        self.emitted = []

    def block(self):
        return build_block(self.c0, self.t, self.win, self.cands, self.W, self.N, self.G, self.Bp)

    def step(self, ids, max_remaining=None):
        """Consume the block's greedy ids.  Returns (emitted tokens, kv moves).

        kv moves are (src, dst) cache-row pairs relative to L before the step;
        after them L grows by len(emitted).
        """
        W, N, G = self.W, self.N, self.G
        ids = [int(x) for x in ids]
        k, m = verify(ids, self.cands, W, N, G)
        out = [ids[0]] + [ids[v_row(W, N, G, k, j)] for j in range(1, m + 1)]
        if max_remaining is not None:
            out = out[:max_remaining]
        e = len(out)
        moves = [(v_row(W, N, G, k, j), j) for j in range(1, e)]
        self.steps += 1
        self.matched_steps += 1 if m >= 1 else 0
        # harvest one new n-gram per window column, then slide the window down
        nl = [ids[la_row(W, N, G, N - 2, c)] for c in range(W)]
        for c in range(W):
            tup = [self.win[r][c] for r in range(1, N - 1)] + [nl[c]]
            self.pool.insert(self.win[0][c], tup)
        self.win = self.win[1:] + [nl]
        self.emitted.extend(out)
        self.t += e
        self.c0 = out[-1]
        self.cands = self.pool.lookup(self.c0)[:G]
        return out, moves


def greedy_lookahead(model, prompt, n_new, W, N, G, Bp=None, seed_pool=True, trace=None):
    """Lookahead decoding on the float64 model; returns (tokens, state)."""
    from . import transformer as tf

    st = LookaheadState(prompt, W, N, G, Bp, seed_pool)
    kv = tf.KVCache(model.shape, len(prompt) + n_new + st.Bp + 1)
    tf.prefill(model, kv, np.asarray(prompt)[:-1])
    while len(st.emitted) < n_new:
        tok, pos, vis = st.block()
        x = tf.forward_block(model, kv, tf.embed(model, tok), pos, vis)
        lg = tf.logits_of(model, x)
        ids = tf.argmax_ids(lg)
        L = kv.L
        if trace is not None:
            trace(dict(L=L, tok=tok, pos=pos, vis=vis, x=x, logits=lg, ids=ids, state=st, kv=kv))
        out, moves = st.step(ids, n_new - len(st.emitted))
        kv.move_rows([(L + s, L + d) for s, d in moves])
        kv.L = L + len(out)
    return np.asarray(st.emitted, dtype=np.int64), st, kv
