"""CPU-only checks of the C-ABI library: it loads, exports every function the header
declares, and its host-side logic (argument checks, block layout) is right."""
import ctypes
import os
import re

import numpy as np
import pytest

from oracle import lookahead as ola

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
LIB = os.path.join(ROOT, "paper_2602_16760_amd", "liblookahead.so")


def declared_functions():
    src = open(os.path.join(ROOT, "include", "la.h")).read()
    src = re.sub(r"/\*.*?\*/", "", src, flags=re.S)
    return sorted(set(re.findall(r"\b(la_[a-z0-9_]+)\s*\(", src)))


def test_library_exports_every_declared_symbol():
    assert os.path.exists(LIB), "build with: python -m paper_2602_16760_amd.build"
    lib = ctypes.CDLL(LIB)
    names = declared_functions()
    assert {"la_init_model", "la_kv_alloc", "la_forward_layers", "la_unembed_argmax", "la_ngram_accept"} <= set(names)
    for n in names:
        assert hasattr(lib, n), f"{n} is declared in la.h but not exported"
    from paper_2602_16760_amd import binding
    assert sorted(binding.EXPORTS) == names


def test_state_struct_layout_matches_header():
    from paper_2602_16760_amd import binding as B
    # 12 int32 + tok/pos (2 x 64 int32) + vis (64 uint64) + win/cand (2 x 64 int32)
    assert B.STATE_BYTES == 12 * 4 + 2 * 64 * 4 + 64 * 8 + 2 * 64 * 4
    assert B.STATE_OFF["vis"] % 8 == 0


@pytest.mark.parametrize("W,N,G,Bp,n_cand", [(2, 3, 1, 7, 1), (4, 3, 4, 32, 2), (5, 4, 5, 32, 5), (7, 4, 7, 48, 0),
                                              (7, 4, 7, 43, 7), (0, 1, 0, 1, 0), (1, 2, 1, 3, 1), (3, 5, 2, 64, 1)])
def test_host_block_layout_matches_oracle(W, N, G, Bp, n_cand):
    from paper_2602_16760_amd import binding as B
    t = 512
    pos, vis = B.la_lookahead_layout(W, N, G, t, n_cand, Bp)
    cands = [tuple(range(N - 1))] * n_cand
    _, opos, ovis = ola.build_block(0, t, [[0] * W for _ in range(max(N - 1, 0))], cands, W, N, G, Bp)
    assert list(pos) == opos
    assert [int(v) for v in vis] == ovis


def test_host_argument_checks():
    from paper_2602_16760_amd import binding as B
    with pytest.raises(B.LaError) as e:
        B.la_lookahead_layout(8, 8, 8, 0, 0, 64)
    assert e.value.code == -1 and "rows" in str(e.value)
    with pytest.raises(B.LaError):
        B.la_lookahead_layout(2, 3, 1, 0, 2, 7)       # n_cand > G
    with pytest.raises(B.LaError):
        B.la_lookahead_layout(2, 3, 1, 0, 1, 6)       # Bp smaller than the block
    with pytest.raises(B.LaError):
        B.la_lookahead_layout(0, 1, 2, 0, 0, 1)       # N=1 needs G=0


@pytest.mark.parametrize("t,n", [(0, 1), (5, 7), (1000, 64), (31, 33)])
def test_host_causal_layout_matches_oracle(t, n):
    """Section 4.4: the plain causal mask of a run of consecutive tokens (prompt chunks)."""
    from paper_2602_16760_amd import binding as B
    pos, vis = B.la_causal_layout(t, n)
    opos, ovis = ola.causal_block(t, n)
    assert list(pos) == list(opos) and [int(v) for v in vis] == [int(v) for v in ovis]
    with pytest.raises(B.LaError):
        B.la_causal_layout(0, 65)
    with pytest.raises(B.LaError):
        B.la_causal_layout(-1, 4)
