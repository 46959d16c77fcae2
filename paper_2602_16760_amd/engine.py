"""Host-side orchestration of the C-ABI calls: model upload, prefill, decode loops.

No arithmetic of the method lives here: every step (embedding gather, layer stack,
unembedding + argmax, n-gram acceptance, KV commit, next-block build) is a library call.
"""
from __future__ import annotations

import time

import numpy as np
import torch

from . import binding as B


class Engine:
    """One model + one KV cache + (optionally) one lookahead controller on cuda:0."""

    def __init__(self, shape, max_len: int, layer_source=None, head: dict | None = None):
        self.shape = shape
        self.max_len = max_len
        head = head or {}
        dev = {k: B.to_device(v) for k, v in head.items()}
        self.model = B.la_init_model(shape, dev.get("embed"), dev.get("g_final"), dev.get("unembed"))
        torch.cuda.synchronize()
        del dev
        if layer_source is not None:
            for l in range(shape.n_layers):
                self.set_layer(l, layer_source(l))
        self.kv = B.la_kv_alloc(self.model, max_len)
        self.pool = None
        self.state = None
        self.la = None

    def set_layer(self, l: int, w: dict):
        dev = {k: B.to_device(v) for k, v in w.items()}
        B.la_model_set_layer(self.model, l, dev)
        torch.cuda.synchronize()  # the library has packed its own copy

    def close(self):
        if self.pool is not None:
            B.la_free_pool(self.pool)
        B.la_free_kv(self.kv)
        B.la_free_model(self.model)
        self.pool = self.kv = self.model = None

    # -- cache ----------------------------------------------------------------------
    def fill_kv(self, layer: int, k: np.ndarray, v: np.ndarray, row0: int = 0):
        kd, vd = B.to_device(k), B.to_device(v)
        B.la_kv_fill(self.kv, layer, row0, kd, vd)
        torch.cuda.synchronize()

    def read_kv(self, layer: int, row0: int, n: int):
        sh = self.shape
        dt = {"f32": torch.float32, "bf16": torch.int16, "f16": torch.float16}[sh.dtype]
        k = torch.empty((n, sh.n_kv_heads, sh.head_dim), dtype=dt, device="cuda")
        v = torch.empty_like(k)
        B.la_kv_read(self.kv, layer, row0, n, k, v)
        torch.cuda.synchronize()
        k, v = k.cpu().numpy(), v.cpu().numpy()
        if sh.dtype == "bf16":
            k, v = k.view(np.uint16), v.view(np.uint16)
        return k, v

    # -- single calls on numpy inputs (tests) -----------------------------------------
    def forward(self, hidden: np.ndarray, pos, vis, layer_begin=0, layer_end=None) -> np.ndarray:
        le = self.shape.n_layers if layer_end is None else layer_end
        h = B.to_device(np.asarray(hidden, dtype=np.float32))
        p = B.to_device(np.asarray(pos, dtype=np.int32))
        m = B.to_device(np.asarray([int(x) for x in vis], dtype=np.uint64))
        B.la_forward_layers(self.model, layer_begin, le, h, p, m, self.kv)
        torch.cuda.synchronize()
        return h.cpu().numpy()

    def unembed_argmax(self, hidden: np.ndarray):
        h = B.to_device(np.asarray(hidden, dtype=np.float32))
        ids = torch.empty(h.shape[0], dtype=torch.int32, device="cuda")
        top2 = torch.empty((h.shape[0], 2), dtype=torch.float32, device="cuda")
        B.la_unembed_argmax(self.model, h, ids, top2)
        torch.cuda.synchronize()
        return ids.cpu().numpy(), top2.cpu().numpy()

    # -- generation -------------------------------------------------------------------
    def prefill(self, tokens: np.ndarray, L0: int = 0):
        """Runs tokens through all layers (la_prefill: causal chunks inside the library); cache rows L0.. are filled."""
        toks = B.to_device(np.asarray(tokens, dtype=np.int32))
        B.la_prefill(self.model, self.kv, toks, L0)
        torch.cuda.synchronize()
        return L0 + len(tokens)

    def start(self, prompt: np.ndarray, W: int, N: int, G: int, Bp: int, seed_pool: bool = True,
              prefill: bool = True):
        """Prefills prompt[:-1] (unless the cache rows are already there) and initialises the
        controller (pool, window, first block)."""
        if self.pool is not None:
            B.la_free_pool(self.pool)
        self.la = (W, N, G)
        self.Bp = Bp
        self.pool = B.la_pool_alloc(self.shape.vocab, N, G)
        self.state = B.new_state()
        if prefill:
            self.prefill(np.asarray(prompt[:-1]))
        B.la_state_init(self.pool, self.kv, W, N, G, B.to_device(np.asarray(prompt, dtype=np.int32)), Bp,
                        seed_pool, self.state)
        torch.cuda.synchronize()
        sh = self.shape
        self._hidden = torch.empty((Bp, sh.d_model), dtype=torch.float32, device="cuda")
        self._ids = torch.empty(Bp, dtype=torch.int32, device="cuda")
        self._top2 = torch.empty((Bp, 2), dtype=torch.float32, device="cuda")
        self._tok = B.state_field(self.state, "tok")[:Bp]
        self._pos = B.state_field(self.state, "pos")[:Bp]
        self._vis = B.state_field(self.state, "vis")[:Bp]

    def step(self, emitted: torch.Tensor, max_total: int):
        """One decode step, enqueued without any host synchronisation."""
        W, N, G = self.la
        sh = self.shape
        B.la_embed(self.model, self._tok, self._hidden)
        B.la_forward_layers(self.model, 0, sh.n_layers, self._hidden, self._pos, self._vis, self.kv)
        B.la_unembed_argmax(self.model, self._hidden, self._ids, self._top2)
        B.la_ngram_accept(self.pool, self.kv, W, N, G, self._ids, self.state, emitted, max_total)

    def generate(self, prompt: np.ndarray, n_new: int, W: int, N: int, G: int, Bp: int | None = None,
                 seed_pool: bool = True, poll: int = 8):
        """Greedy generation; {W=0, N=1, G=0} is sequential decoding.  Returns (tokens, stats)."""
        rows = 1 + (W + G) * (N - 1)
        Bp = rows if Bp is None else Bp
        self.start(prompt, W, N, G, Bp, seed_pool)
        emitted = torch.zeros(n_new, dtype=torch.int32, device="cuda")
        n_field = B.state_field(self.state, "n_emitted")
        done = 0
        while done < n_new:
            for _ in range(poll):
                self.step(emitted, n_new)
            done = int(n_field.item())
        st = B.read_state(self.state)
        if st.error:
            raise B.LaError(-4 if st.error & 4 else -3, f"a kernel raised error word {st.error} during generation")
        return emitted.cpu().numpy().astype(np.int64), dict(steps=st.steps, matched_steps=st.matched_steps,
                                                            n_emitted=st.n_emitted, L=st.L)

    # -- the split deployment on one GPU, with an injected round trip ---------------------------------
    def step_split(self, emitted: torch.Tensor, max_total: int, head_layers: int, tail_layers: int, rtt_ms: float):
        """One decode step cut where the paper cuts the model (Section 3.1): the first
        `head_layers` and the last `tail_layers` layers are the local half, the layers between
        them the cloud half; the hidden states cross the cut twice per step, and each crossing
        costs half of rtt_ms here (a host sleep after the stream has drained, as a network would
        make the next half wait).  Returns (local_ms, cloud_ms) of GPU time, by host clock."""
        W, N, G = self.la
        n = self.shape.n_layers
        t0 = time.perf_counter()
        B.la_embed(self.model, self._tok, self._hidden)
        B.la_forward_layers(self.model, 0, head_layers, self._hidden, self._pos, self._vis, self.kv)
        torch.cuda.synchronize()
        t1 = time.perf_counter()
        time.sleep(rtt_ms / 2000.0)
        t2 = time.perf_counter()
        B.la_forward_layers(self.model, head_layers, n - tail_layers, self._hidden, self._pos, self._vis, self.kv)
        torch.cuda.synchronize()
        t3 = time.perf_counter()
        time.sleep(rtt_ms / 2000.0)
        t4 = time.perf_counter()
        B.la_forward_layers(self.model, n - tail_layers, n, self._hidden, self._pos, self._vis, self.kv)
        B.la_unembed_argmax(self.model, self._hidden, self._ids, self._top2)
        B.la_ngram_accept(self.pool, self.kv, W, N, G, self._ids, self.state, emitted, max_total)
        torch.cuda.synchronize()
        t5 = time.perf_counter()
        return ((t1 - t0) + (t5 - t4)) * 1e3, (t3 - t2) * 1e3

    def generate_split(self, prompt: np.ndarray, n_new: int, W: int, N: int, G: int, head_layers: int, tail_layers: int,
                       rtt_ms: float, Bp: int | None = None, seed_pool: bool = True):
        """Greedy generation through step_split.  Returns (tokens, stats): steps, tokens per
        step, wall milliseconds per step, local and cloud GPU milliseconds per step, and the
        measured throughput, from which la_rtt_fixed_overhead / la_rtt_project give the paper's
        decomposition and projection (Section 6.3)."""
        rows = 1 + (W + G) * (N - 1)
        Bp = rows if Bp is None else Bp
        self.start(prompt, W, N, G, Bp, seed_pool)
        emitted = torch.zeros(n_new, dtype=torch.int32, device="cuda")
        n_field = B.state_field(self.state, "n_emitted")
        steps, local, cloud = 0, 0.0, 0.0
        t0 = time.perf_counter()
        while int(n_field.item()) < n_new:
            l, c = self.step_split(emitted, n_new, head_layers, tail_layers, rtt_ms)
            local += l
            cloud += c
            steps += 1
        wall = (time.perf_counter() - t0) * 1e3
        st = B.read_state(self.state)
        if st.error:
            raise B.LaError(-4 if st.error & 4 else -3, f"a kernel raised error word {st.error} during generation")
        return emitted.cpu().numpy().astype(np.int64), dict(
            steps=steps, tokens_per_step=n_new / steps, ms_per_step=wall / steps, local_ms=local / steps,
            cloud_ms=cloud / steps, tok_per_s=n_new / (wall / 1e3), matched_steps=st.matched_steps)

    # -- Jacobi decoding (Section 4.2) ------------------------------------------------------------------
    def generate_jacobi(self, prompt: np.ndarray, n_new: int, k: int, Bp: int | None = None, poll: int = 8):
        """Greedy generation by Jacobi iteration on blocks of k positions.  Returns (tokens, stats):
        passes (each one network round trip in the split deployment), blocks committed, tokens per pass."""
        Bp = k if Bp is None else Bp
        sh = self.shape
        self.state = B.new_state()
        self.prefill(np.asarray(prompt[:-1]))
        B.la_jacobi_init(self.kv, k, B.to_device(np.asarray(prompt, dtype=np.int32)), Bp, self.state)
        hidden = torch.empty((Bp, sh.d_model), dtype=torch.float32, device="cuda")
        ids = torch.empty(Bp, dtype=torch.int32, device="cuda")
        tok = B.state_field(self.state, "tok")[:Bp]
        pos = B.state_field(self.state, "pos")[:Bp]
        vis = B.state_field(self.state, "vis")[:Bp]
        emitted = torch.zeros(n_new, dtype=torch.int32, device="cuda")
        n_field = B.state_field(self.state, "n_emitted")
        done = 0
        while done < n_new:
            for _ in range(poll):
                B.la_embed(self.model, tok, hidden)
                B.la_forward_layers(self.model, 0, sh.n_layers, hidden, pos, vis, self.kv)
                B.la_unembed_argmax(self.model, hidden, ids)
                B.la_jacobi_accept(self.kv, k, ids, self.state, emitted, n_new)
            done = int(n_field.item())
        st = B.read_state(self.state)
        if st.error:
            raise B.LaError(-4 if st.error & 4 else -3, f"a kernel raised error word {st.error} during generation")
        return emitted.cpu().numpy().astype(np.int64), dict(passes=st.steps, blocks=st.matched_steps, n_emitted=st.n_emitted,
                                                            L=st.L, tokens_per_pass=n_new / max(st.steps, 1))
