"""Jacobi parallel decoding (Section 4.2), integer logic and the float64 decode loop.

TEST INFRASTRUCTURE ONLY (see the package header).

A block of k future positions is guessed, all k positions go through one forward pass under
the plain causal mask of Section 4.4 (row i sees the committed cache and block rows <= i), and
every position's guess is replaced by the model's greedy prediction for it; this repeats until
the guesses no longer change, and the converged block commits k tokens.  Rows: row 0 carries the
last committed token c0 at position t, row i >= 1 carries the current guess y_i for position
t + i, i < k; the prediction at row i is the new guess for y_{i+1}, i.e. the k predictions are
the new y_1..y_k.

Readings (the paper gives the method in two sentences):
  * the first guess of every position of a block is the last committed token;
  * a block has converged when an iteration returns the guesses it was given, and after k
    iterations at the latest: iteration j fixes y_j for good (its row saw only c0 and y_1..y_{j-1},
    which were already final), so k iterations always reach the greedy continuation;
  * "iterations" counts forward passes, each of which is one network round trip (Section 4.2's
    throughput relation tok/s = k / (iterations * RTT)).
"""
import numpy as np

from .lookahead import causal_block


class JacobiState:
    """Controller state between iterations; `step(ids)` consumes one pass's greedy ids."""

    def __init__(self, prompt, k, Bp=None):
        prompt = [int(x) for x in prompt]
        assert k >= 1
        self.k = k
        self.Bp = k if Bp is None else Bp
        assert self.Bp >= k
        self.t = len(prompt) - 1      # position of c0 = committed cache length L
        self.c0 = prompt[-1]
        self.y = [self.c0] * k        # guesses y_1..y_k
        self.it = 0                   # iterations spent on the current block
        self.iterations = 0           # forward passes in total
        self.blocks = 0               # blocks committed
        self.last_iterations = 0      # iterations the last committed block took
        self.emitted = []

    def block(self):
        """(tokens, positions, visibility masks) of the next pass, padded to Bp rows that see only themselves."""
        k, Bp = self.k, self.Bp
        pos, vis = causal_block(self.t, k)
        tok = [self.c0] + self.y[:k - 1]
        tok += [0] * (Bp - k)
        pos += [self.t + k - 1] * (Bp - k)
        vis += [1 << b for b in range(k, Bp)]
        return tok, pos, vis

    def step(self, ids, max_remaining=None):
        """Returns the tokens committed by this pass ([] while the block is still moving)."""
        k = self.k
        new = [int(x) for x in ids[:k]]
        self.it += 1
        self.iterations += 1
        done = new == self.y or self.it == k
        self.y = new
        if not done:
            return []
        out = list(new)
        if max_remaining is not None:
            out = out[:max_remaining]
        self.emitted.extend(out)
        self.t += len(out)            # the pass's cache rows t..t+e-1 came from the final tokens: they stay
        self.c0 = out[-1]
        self.y = [self.c0] * k
        self.blocks += 1
        self.last_iterations = self.it
        self.it = 0
        return out


def greedy_jacobi(model, prompt, n_new, k, Bp=None):
    """Jacobi decoding on the float64 model; returns (tokens, state, cache)."""
    from . import transformer as tf

    st = JacobiState(prompt, k, Bp)
    kv = tf.KVCache(model.shape, len(prompt) + n_new + st.Bp + 1)
    tf.prefill(model, kv, np.asarray(prompt)[:-1])
    while len(st.emitted) < n_new:
        tok, pos, vis = st.block()
        x = tf.forward_block(model, kv, tf.embed(model, tok), pos, vis)
        ids = tf.argmax_ids(tf.logits_of(model, x))
        out = st.step(ids, n_new - len(st.emitted))
        kv.L += len(out)
    return np.asarray(st.emitted, dtype=np.int64), st, kv
