"""la_unembed_argmax_noalloc, the entry point for callers that cannot allocate device memory,
against la_unembed_argmax through the C-ABI: the same kernel on a static scratch array must give
the same bits.  Two calls in a row share the array, the second with fewer rows (its first rows
are then checked against a scratch that still holds the larger call's words), then a second,
smaller model on the same array, and the sizes beyond the array's limits are refused."""
import numpy as np
import pytest

import synth
from gpu_util import gpu_engine

pytestmark = pytest.mark.gpu


def _both(eng, x):
    import torch
    from paper_2602_16760_amd import binding as B
    h = B.to_device(np.asarray(x, dtype=np.float32))
    out = []
    for fn in (B.la_unembed_argmax, B.la_unembed_argmax_noalloc):
        ids = torch.full((h.shape[0],), -7, dtype=torch.int32, device="cuda")
        top2 = torch.full((h.shape[0], 2), float("nan"), dtype=torch.float32, device="cuda")
        fn(eng.model, h, ids, top2)
        torch.cuda.synchronize()
        out.append((ids.cpu().numpy(), top2.cpu().numpy()))
    return out


def test_noalloc_unembed_equals_unembed_on_two_calls_in_a_row():
    import torch
    from paper_2602_16760_amd import binding as B
    shape = synth.SHAPES["small_bf16"].with_layers(1)
    eng = gpu_engine(shape, 64, seed=7)
    small = gpu_engine(synth.SHAPES["small64_bf16"].with_layers(1), 64, seed=3)
    try:
        for Bp, seed in ((48, 8), (17, 9)):  # the second call is the smaller one
            x = synth.hidden_block(shape, Bp, seed) * 3.0
            (ids, top2), (ids_na, top2_na) = _both(eng, x)
            assert ids.min() >= 0 and ids.max() < shape.vocab
            assert np.array_equal(ids_na, ids), f"Bp={Bp}"
            assert np.array_equal(top2_na.view(np.uint32), top2.view(np.uint32)), f"Bp={Bp}"
        # another model, other sizes, same array
        x = synth.hidden_block(small.shape, 5, 10)
        (ids, top2), (ids_na, top2_na) = _both(small, x)
        assert np.array_equal(ids_na, ids) and np.array_equal(top2_na.view(np.uint32), top2.view(np.uint32))
        # no device memory is taken from torch's allocator or the driver by the call itself
        h = B.to_device(synth.hidden_block(shape, 32, 11).astype(np.float32))
        ids_t = torch.empty(32, dtype=torch.int32, device="cuda")
        torch.cuda.synchronize()
        free0, _ = torch.cuda.mem_get_info()
        stats0 = torch.cuda.memory_allocated()
        for _ in range(3):
            B.la_unembed_argmax_noalloc(eng.model, h, ids_t)
        torch.cuda.synchronize()
        assert torch.cuda.mem_get_info()[0] == free0 and torch.cuda.memory_allocated() == stats0
    finally:
        eng.close()
        small.close()


def test_noalloc_unembed_refuses_what_the_array_cannot_hold():
    from paper_2602_16760_amd import binding as B
    import torch
    f32 = gpu_engine(synth.SHAPES["tiny_f32"].with_layers(1), 8, seed=1)
    try:
        h = B.to_device(synth.hidden_block(f32.shape, 4, 1).astype(np.float32))
        ids = torch.empty(4, dtype=torch.int32, device="cuda")
        with pytest.raises(RuntimeError, match="matrix-core"):
            B.la_unembed_argmax_noalloc(f32.model, h, ids)
    finally:
        f32.close()
    # a vocabulary beyond the partial-record limit (one layer, narrow model: 67 MB of unembedding)
    import dataclasses
    wide = dataclasses.replace(synth.SHAPES["small64_bf16"].with_layers(1), vocab=65536 + 4096)
    eng = gpu_engine(wide, 8, seed=2)
    try:
        h = B.to_device(synth.hidden_block(wide, 4, 2).astype(np.float32))
        ids = torch.empty(4, dtype=torch.int32, device="cuda")
        B.la_unembed_argmax(eng.model, h, ids)  # the allocating entry point takes it
        torch.cuda.synchronize()
        with pytest.raises(RuntimeError, match="partial arg-max records"):
            B.la_unembed_argmax_noalloc(eng.model, h, ids)
    finally:
        eng.close()
