"""GPU parity at the benchmark's full size and launch configuration.

Mistral-7B-shaped 30-layer stack, bf16, KV cache pre-filled to 512 rows, the 32-row lookahead
block (W=5, N=4, G=5) -- the workload bench.py times -- run as ONE la_forward_layers call, then
la_unembed_argmax, against the float64 oracle on the same seeded inputs.  The oracle walks the
stack one layer at a time on the arrays that are uploaded to the GPU (13 GB of weights are never
held twice), and checks every row of the block, not a sample: one layer of 32 rows is a fraction
of a second of float64 numpy.

Bars (the benchmark spec): hidden states within max relative error 2e-2 per row
(max|gpu - oracle| / max|oracle|); ids bit-exact wherever the top-1/top-2 margin exceeds 1e-2,
and within that margin of the best elsewhere.  The arg-max is decided by both sides on the same
hidden states (the GPU's): through 30 bf16 layers the hidden-state bar itself allows logit changes
far above 1e-2, so end to end the ids are required to agree where the oracle's margin is clear of
the measured logit change as well.
"""
import os
import sys
import time
from concurrent.futures import ThreadPoolExecutor

import numpy as np
import pytest

import synth
from oracle import lookahead as ola
from oracle import transformer as otf
from tests.gpu_util import row_rel_err

pytestmark = pytest.mark.gpu

W, N, G, BP, L0, N_LAYERS = 5, 4, 5, 32, 512, 30


def _say(*a):
    print("[fullsize]", *a, file=sys.stderr, flush=True)


def test_config2_full_stack_matches_oracle():
    from paper_2602_16760_amd import binding as B
    from paper_2602_16760_amd.engine import Engine

    t0 = time.time()
    shape = synth.SHAPES["mistral7b"].with_layers(N_LAYERS)
    head = synth.head_weights(shape, 0, unit_gains=False)
    eng = Engine(shape, L0 + BP, None, head)
    okv = otf.KVCache(shape, L0 + BP)
    _, pos, vis = ola.build_block(0, L0, [[0] * W for _ in range(N - 1)], [(0,) * (N - 1)] * 3, W, N, G, BP)
    x = synth.hidden_block(shape, BP, 5)
    want = x.astype(np.float64)
    holder = {}
    om = otf.Model(shape, lambda l: holder[l], head, cache=False)
    try:
        # gains drawn from U(0.5, 1.5): a dropped or misplaced gain fails the comparison
        with ThreadPoolExecutor(max_workers=min(8, os.cpu_count() or 8)) as ex:
            futs = [ex.submit(synth.layer_weights, shape, l, 0, False) for l in range(N_LAYERS)]
            for l in range(N_LAYERS):
                w = futs[l].result()
                futs[l] = None
                eng.set_layer(l, w)
                k, v = synth.kv_fill(shape, l, L0, 0)
                eng.fill_kv(l, k, v)
                okv.fill(l, k, v)
                okv.L = L0
                holder[l] = w
                want = otf.forward_block(om, okv, want, pos, vis, l, l + 1)
                del holder[l]
                if l % 5 == 4:
                    _say(f"layer {l + 1}/{N_LAYERS} uploaded and walked by the oracle ({time.time() - t0:.0f} s)")
        B.la_kv_set_len(eng.kv, L0)
        got = eng.forward(x, pos, vis)  # all 30 layers in one call, as in bench.py
        err = row_rel_err(got, want)
        _say(f"hidden: max row rel err {err.max():.3e} (rows: {np.array2string(err, precision=4)})")
        assert np.all(np.isfinite(got))
        assert err.max() <= 2e-2
        # the block's K, V of the last layer landed in cache rows L..L+Bp-1
        k, v = eng.read_kv(N_LAYERS - 1, L0, BP)
        kf, vf = synth.bf16_to_f32(k), synth.bf16_to_f32(v)
        ko, vo = okv.K[N_LAYERS - 1, L0:L0 + BP], okv.V[N_LAYERS - 1, L0:L0 + BP]
        # (stored as bf16: the hidden-state bar plus one bf16 rounding of the stored value, 2^-8)
        kv_tol = 2e-2 + 2.0 ** -8
        assert np.max(np.abs(kf - ko)) / np.max(np.abs(ko)) <= kv_tol
        assert np.max(np.abs(vf - vo)) / np.max(np.abs(vo)) <= kv_tol
        # greedy ids of every row from the GPU's own hidden states against the oracle's logits
        lg = otf.logits_of(om, want)
        t1, t2 = otf.top2_margin(lg)
        ids, top2 = eng.unembed_argmax(got)
        safe = (t1 - t2) > 1e-2
        lg_gpu_hidden = otf.logits_of(om, got.astype(np.float64))  # isolates the unembedding from the stack's error
        ids_ref = otf.argmax_ids(lg_gpu_hidden)
        g1, g2 = otf.top2_margin(lg_gpu_hidden)
        safe_u = (g1 - g2) > 1e-2
        _say(f"ids: {int(safe_u.sum())}/{BP} rows with margin > 1e-2; equal on all of them: "
             f"{bool(np.array_equal(ids[safe_u], ids_ref[safe_u]))}")
        assert np.array_equal(ids[safe_u], ids_ref[safe_u])
        for b in np.where(~safe_u)[0]:
            assert g1[b] - lg_gpu_hidden[b, ids[b]] <= 1e-2
        # end to end (stack + unembedding): the emitted id is the oracle's wherever the oracle's
        # margin is clear of the stack's bf16 error as well
        clear = (t1 - t2) > 1e-2 + 2 * np.max(np.abs(lg - lg_gpu_hidden), axis=-1)
        assert np.array_equal(ids[clear], otf.argmax_ids(lg)[clear])
        _say(f"end to end: {int(clear.sum())}/{BP} rows clear of the stack's error, all equal; "
             f"{int(safe.sum())} rows have an oracle margin > 1e-2")
        # (Rows whose oracle margin lies between 1e-2 and the logit change that the allowed hidden
        # error itself causes may differ end to end: the two bars cannot both bind there.  The
        # arg-max decision is compared on the same hidden states above, as the bar on ids asks.)
        n_same = int(np.sum(ids[safe] == otf.argmax_ids(lg)[safe]))
        _say(f"end to end on rows with an oracle margin > 1e-2: {n_same}/{int(safe.sum())} ids equal")
        # run-to-run bit stability at full size
        again = eng.forward(x, pos, vis)
        assert np.array_equal(got, again)
    finally:
        eng.close()
