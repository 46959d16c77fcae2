"""ctypes binding of liblookahead.so: argument marshalling only.

The functions carry the C names (la_init_model, la_kv_alloc, la_forward_layers,
la_unembed_argmax, la_ngram_accept, ...).  torch is used for device memory and
streams; every step of the path runs inside the library's kernels.  Importing
this module fails loudly when the library has not been built.
"""
from __future__ import annotations

import ctypes as C
import os

import numpy as np
import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "liblookahead.so")

LA_MAX_ROWS = 64
LA_F32, LA_BF16, LA_F16 = 0, 1, 2


class LaError(RuntimeError):
    def __init__(self, code, text):
        super().__init__(f"liblookahead error {code}: {text}")
        self.code = code


class la_model_desc(C.Structure):
    _fields_ = [(n, C.c_int32) for n in
                ("n_layers", "d_model", "n_q_heads", "n_kv_heads", "head_dim", "d_ffn", "vocab")] + \
               [("rms_eps", C.c_float), ("rope_theta", C.c_float), ("dtype", C.c_int32)]


class la_layer_weights(C.Structure):
    _fields_ = [(n, C.c_void_p) for n in
                ("wq", "wk", "wv", "wo", "wgate", "wup", "wdown", "g_attn", "g_mlp")]


class la_lookahead_desc(C.Structure):
    _fields_ = [("W", C.c_int32), ("N", C.c_int32), ("G", C.c_int32)]


class la_step_state(C.Structure):
    _fields_ = [(n, C.c_int32) for n in
                ("L", "c0", "n_cand", "Bp", "steps", "matched_steps", "n_emitted", "last_emitted",
                 "last_k", "last_m", "error", "reserved")] + \
               [("tok", C.c_int32 * LA_MAX_ROWS), ("pos", C.c_int32 * LA_MAX_ROWS),
                ("vis", C.c_uint64 * LA_MAX_ROWS), ("win", C.c_int32 * LA_MAX_ROWS),
                ("cand", C.c_int32 * LA_MAX_ROWS)]


class la_profile_entry(C.Structure):
    _fields_ = [("name", C.c_char * 48), ("launches", C.c_int32), ("total_ms", C.c_float)]


STATE_BYTES = C.sizeof(la_step_state)
STATE_OFF = {n: getattr(la_step_state, n).offset for n, _ in la_step_state._fields_}

EXPORTS = [
    "la_init_model", "la_model_set_layer", "la_free_model", "la_kv_alloc", "la_kv_set_len", "la_kv_get_len",
    "la_kv_fill", "la_kv_read", "la_free_kv", "la_embed", "la_forward_layers", "la_unembed_argmax",
    "la_unembed_argmax_noalloc", "la_causal_layout", "la_set_barrier_timeout",
    "la_prefill", "la_jacobi_init", "la_jacobi_accept", "la_rtt_fixed_overhead", "la_rtt_project", "la_jacobi_project",
    "la_pool_alloc", "la_free_pool", "la_state_init", "la_ngram_accept", "la_lookahead_layout",
    "la_profile_enable", "la_profile_select", "la_profile_read", "la_profile_copy", "la_last_error",
]


def _load():
    if not os.path.exists(LIB_PATH):
        raise ImportError(
            f"{LIB_PATH} is missing: build it with `python -m paper_2602_16760_amd.build` "
            "(there is no fallback path)")
    lib = C.CDLL(LIB_PATH)
    vp, i32, f32 = C.c_void_p, C.c_int, C.c_float
    sig = {
        "la_init_model": (i32, [C.POINTER(la_model_desc), C.POINTER(la_layer_weights), vp, vp, vp, vp, C.POINTER(vp)]),
        "la_model_set_layer": (i32, [vp, i32, C.POINTER(la_layer_weights), vp]),
        "la_free_model": (None, [vp]),
        "la_kv_alloc": (i32, [vp, i32, C.POINTER(vp)]),
        "la_kv_set_len": (i32, [vp, i32, vp]),
        "la_kv_get_len": (i32, [vp, C.POINTER(i32), vp]),
        "la_kv_fill": (i32, [vp, i32, i32, vp, vp, i32, vp]),
        "la_kv_read": (i32, [vp, i32, i32, i32, vp, vp, vp]),
        "la_free_kv": (None, [vp]),
        "la_embed": (i32, [vp, vp, i32, vp, vp]),
        "la_forward_layers": (i32, [vp, i32, i32, vp, i32, vp, vp, vp, vp]),
        "la_unembed_argmax": (i32, [vp, vp, i32, vp, vp, vp]),
        "la_unembed_argmax_noalloc": (i32, [vp, vp, i32, vp, vp, vp]),
        "la_pool_alloc": (i32, [i32, i32, i32, C.POINTER(vp)]),
        "la_free_pool": (None, [vp]),
        "la_state_init": (i32, [vp, vp, C.POINTER(la_lookahead_desc), vp, i32, i32, i32, vp, vp]),
        "la_ngram_accept": (i32, [vp, vp, C.POINTER(la_lookahead_desc), vp, vp, vp, i32, vp]),
        "la_prefill": (i32, [vp, vp, vp, i32, i32, vp]),
        "la_jacobi_init": (i32, [vp, i32, vp, i32, i32, vp, vp]),
        "la_jacobi_accept": (i32, [vp, i32, vp, vp, vp, i32, vp]),
        "la_lookahead_layout": (i32, [C.POINTER(la_lookahead_desc), i32, i32, i32, C.POINTER(C.c_int32), C.POINTER(C.c_uint64)]),
        "la_causal_layout": (i32, [i32, i32, C.POINTER(C.c_int32), C.POINTER(C.c_uint64)]),
        "la_set_barrier_timeout": (i32, [vp, C.c_uint]),
        "la_rtt_fixed_overhead": (i32, [C.c_double, C.c_double, C.POINTER(C.c_double)]),
        "la_rtt_project": (i32, [C.c_double, C.c_double, C.c_double, C.POINTER(C.c_double)]),
        "la_jacobi_project": (i32, [i32, C.c_double, C.c_double, C.POINTER(C.c_double)]),
        "la_profile_enable": (i32, [i32]),
        "la_profile_select": (i32, [C.c_char_p]),
        "la_profile_read": (i32, [C.POINTER(la_profile_entry), i32]),
        "la_profile_copy": (i32, [C.c_void_p, C.c_void_p, C.c_size_t, C.c_void_p]),
        "la_last_error": (C.c_char_p, []),
    }
    for name, (res, args) in sig.items():
        fn = getattr(lib, name)
        fn.restype = res
        fn.argtypes = args
    return lib


lib = _load()


def _check(rc):
    if rc != 0:
        raise LaError(rc, lib.la_last_error().decode())


def _stream(stream=None):
    s = torch.cuda.current_stream() if stream is None else stream
    return C.c_void_p(s.cuda_stream)


def _ptr(t):
    if t is None:
        return C.c_void_p(0)
    assert t.is_cuda and t.is_contiguous(), "device pointer arguments must be contiguous CUDA tensors"
    return C.c_void_p(t.data_ptr())


def to_device(a: np.ndarray) -> torch.Tensor:
    """numpy array -> device tensor with the same bytes (uint16/uint64 travel as int16/int64)."""
    a = np.ascontiguousarray(a)
    if a.dtype == np.uint16:
        a = a.view(np.int16)
    elif a.dtype == np.uint64:
        a = a.view(np.int64)
    elif a.dtype == np.uint32:
        a = a.view(np.int32)
    return torch.from_numpy(a).cuda()


def make_desc(shape) -> la_model_desc:
    return la_model_desc(shape.n_layers, shape.d_model, shape.n_q_heads, shape.n_kv_heads, shape.head_dim,
                         shape.d_ffn, shape.vocab, shape.rms_eps, shape.rope_theta,
                         {"f32": LA_F32, "bf16": LA_BF16, "f16": LA_F16}[shape.dtype])


def _layer_struct(w: dict) -> la_layer_weights:
    return la_layer_weights(*[_ptr(w[k]) for k in ("wq", "wk", "wv", "wo", "wgate", "wup", "wdown", "g_attn", "g_mlp")])


# ---- thin wrappers, one per C entry point ---------------------------------------------
def la_init_model(shape, embed=None, g_final=None, unembed=None, stream=None):
    """Creates an empty model (layers are added with la_model_set_layer).  Returns the handle."""
    out = C.c_void_p()
    d = make_desc(shape)
    _check(lib.la_init_model(C.byref(d), None, _ptr(embed), _ptr(g_final), _ptr(unembed), _stream(stream), C.byref(out)))
    return out


def la_model_set_layer(model, layer: int, w: dict, stream=None):
    s = _layer_struct(w)
    _check(lib.la_model_set_layer(model, layer, C.byref(s), _stream(stream)))


def la_free_model(model):
    lib.la_free_model(model)


def la_kv_alloc(model, max_len: int):
    out = C.c_void_p()
    _check(lib.la_kv_alloc(model, max_len, C.byref(out)))
    return out


def la_kv_set_len(kv, L: int, stream=None):
    _check(lib.la_kv_set_len(kv, L, _stream(stream)))


def la_kv_get_len(kv, stream=None) -> int:
    v = C.c_int(0)
    _check(lib.la_kv_get_len(kv, C.byref(v), _stream(stream)))
    return v.value


def la_kv_fill(kv, layer, row0, k, v, stream=None):
    _check(lib.la_kv_fill(kv, layer, row0, _ptr(k), _ptr(v), k.shape[0], _stream(stream)))


def la_kv_read(kv, layer, row0, n, k_out, v_out, stream=None):
    _check(lib.la_kv_read(kv, layer, row0, n, _ptr(k_out), _ptr(v_out), _stream(stream)))


def la_free_kv(kv):
    lib.la_free_kv(kv)


def la_embed(model, tok, hidden, stream=None):
    _check(lib.la_embed(model, _ptr(tok), hidden.shape[0], _ptr(hidden), _stream(stream)))


def la_forward_layers(model, layer_begin, layer_end, hidden, pos, vis, kv, stream=None):
    assert hidden.dtype == torch.float32 and pos.dtype == torch.int32 and vis.dtype == torch.int64
    _check(lib.la_forward_layers(model, layer_begin, layer_end, _ptr(hidden), hidden.shape[0], _ptr(pos), _ptr(vis),
                                 kv, _stream(stream)))


def la_unembed_argmax(model, hidden, ids, top2=None, stream=None):
    assert ids.dtype == torch.int32
    _check(lib.la_unembed_argmax(model, _ptr(hidden), hidden.shape[0], _ptr(ids), _ptr(top2), _stream(stream)))


def la_unembed_argmax_noalloc(model, hidden, ids, top2=None, stream=None):
    assert ids.dtype == torch.int32
    _check(lib.la_unembed_argmax_noalloc(model, _ptr(hidden), hidden.shape[0], _ptr(ids), _ptr(top2), _stream(stream)))


def la_pool_alloc(vocab, N, G):
    out = C.c_void_p()
    _check(lib.la_pool_alloc(vocab, N, G, C.byref(out)))
    return out


def la_free_pool(pool):
    lib.la_free_pool(pool)


def la_state_init(pool, kv, W, N, G, prompt, Bp, seed_pool, state, stream=None):
    d = la_lookahead_desc(W, N, G)
    _check(lib.la_state_init(pool, kv, C.byref(d), _ptr(prompt), prompt.shape[0], Bp, int(seed_pool), _ptr(state),
                             _stream(stream)))


def la_ngram_accept(pool, kv, W, N, G, ids, state, emitted, max_total, stream=None):
    d = la_lookahead_desc(W, N, G)
    _check(lib.la_ngram_accept(pool, kv, C.byref(d), _ptr(ids), _ptr(state), _ptr(emitted), max_total, _stream(stream)))


def la_prefill(model, kv, tok, L0=0, stream=None):
    assert tok.dtype == torch.int32
    _check(lib.la_prefill(model, kv, _ptr(tok), tok.shape[0], L0, _stream(stream)))


def la_jacobi_init(kv, k, prompt, Bp, state, stream=None):
    _check(lib.la_jacobi_init(kv, k, _ptr(prompt), prompt.shape[0], Bp, _ptr(state), _stream(stream)))


def la_jacobi_accept(kv, k, ids, state, emitted, max_total, stream=None):
    _check(lib.la_jacobi_accept(kv, k, _ptr(ids), _ptr(state), _ptr(emitted), max_total, _stream(stream)))


def la_lookahead_layout(W, N, G, t, n_cand, Bp):
    """Host helper -> (pos int32[Bp], vis uint64[Bp]) numpy arrays."""
    d = la_lookahead_desc(W, N, G)
    pos = (C.c_int32 * Bp)()
    vis = (C.c_uint64 * Bp)()
    _check(lib.la_lookahead_layout(C.byref(d), t, n_cand, Bp, pos, vis))
    return np.array(pos, dtype=np.int32), np.array(vis, dtype=np.uint64)


def la_causal_layout(t, n):
    """Host helper -> (pos int32[n], vis uint64[n]) numpy arrays of a causal block of n tokens at position t."""
    pos = (C.c_int32 * n)()
    vis = (C.c_uint64 * n)()
    _check(lib.la_causal_layout(t, n, pos, vis))
    return np.array(pos, dtype=np.int32), np.array(vis, dtype=np.uint64)


def la_set_barrier_timeout(model, polls):
    _check(lib.la_set_barrier_timeout(model, polls))


def la_rtt_fixed_overhead(per_step_ms, rtt_ms) -> float:
    out = C.c_double(0.0)
    _check(lib.la_rtt_fixed_overhead(per_step_ms, rtt_ms, C.byref(out)))
    return out.value


def la_rtt_project(tokens_per_step, rtt_ms, fixed_ms) -> float:
    out = C.c_double(0.0)
    _check(lib.la_rtt_project(tokens_per_step, rtt_ms, fixed_ms, C.byref(out)))
    return out.value


def la_jacobi_project(k, iterations, rtt_ms) -> float:
    out = C.c_double(0.0)
    _check(lib.la_jacobi_project(k, iterations, rtt_ms, C.byref(out)))
    return out.value


def la_profile_enable(on: bool):
    _check(lib.la_profile_enable(int(on)))


def la_profile_select(name):
    _check(lib.la_profile_select(name.encode() if name else None))


def la_profile_read(cap=64):
    buf = (la_profile_entry * cap)()
    n = lib.la_profile_read(buf, cap)
    return {buf[i].name.decode(): (buf[i].launches, buf[i].total_ms) for i in range(n)}


def la_profile_copy(dst: torch.Tensor, src: torch.Tensor):
    _check(lib.la_profile_copy(dst.data_ptr(), src.data_ptr(), src.numel() * src.element_size(), _stream()))


# ---- state helpers (views of the published struct layout) ------------------------------
def new_state() -> torch.Tensor:
    return torch.zeros(STATE_BYTES, dtype=torch.uint8, device="cuda")


def state_field(state: torch.Tensor, name: str) -> torch.Tensor:
    """Device view of one field of la_step_state (no copy)."""
    off = STATE_OFF[name]
    if name == "vis":
        return state[off:off + 8 * LA_MAX_ROWS].view(torch.int64)
    if name in ("tok", "pos", "win", "cand"):
        return state[off:off + 4 * LA_MAX_ROWS].view(torch.int32)
    return state[off:off + 4].view(torch.int32)


def read_state(state: torch.Tensor) -> la_step_state:
    raw = bytes(state.cpu().numpy().tobytes())
    return la_step_state.from_buffer_copy(raw)
