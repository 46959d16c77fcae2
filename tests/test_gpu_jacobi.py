"""Jacobi decoding (Section 4.2) on the GPU against the oracle's controller and decode loop."""
import numpy as np
import pytest

import synth
from gpu_util import gpu_engine, oracle_model
from oracle import jacobi as ojc
from oracle import transformer as otf

pytestmark = pytest.mark.gpu
MARGIN = 1e-2


@pytest.mark.parametrize("k,Bp,V", [(1, 1, 16), (4, 4, 32), (5, 8, 9), (16, 17, 12), (64, 64, 5)])
def test_jacobi_controller_state_is_bit_exact(k, Bp, V):
    """Integer-level parity: both controllers get the same ids; every state word is compared.
    The ids come from a rule that converges early on some blocks and only at pass k on others."""
    import torch
    from paper_2602_16760_amd import binding as B
    shape = synth.SHAPES["tiny_f32"].with_layers(1)
    eng = gpu_engine(shape, 4096, seed=0, head=False)
    rng = np.random.default_rng(k * 100 + V)
    prompt = rng.integers(0, V, size=20).astype(np.int32)
    n_total = 3 * k + 200
    try:
        state = B.new_state()
        B.la_jacobi_init(eng.kv, k, B.to_device(prompt), Bp, state)
        ost = ojc.JacobiState(prompt, k, Bp)
        emitted = torch.zeros(n_total, dtype=torch.int32, device="cuda")
        passes = 0
        while len(ost.emitted) < n_total:
            st = B.read_state(state)
            tok, pos, vis = ost.block()
            assert list(st.tok[:Bp]) == tok and list(st.pos[:Bp]) == pos and list(st.vis[:Bp]) == vis
            assert st.L == ost.t and st.c0 == ost.c0 and st.n_cand == k and st.Bp == Bp
            assert list(st.cand[:k]) == ost.y and st.last_k == ost.it
            mode = passes % 7
            if mode < 3:        # return the input: converged
                ids = np.asarray(ost.y + [0] * (Bp - k), dtype=np.int32)
            elif mode < 5:      # a successor rule: one more position settles per pass
                ids = np.asarray([(t + 1) % V for t in tok[:k]] + [0] * (Bp - k), dtype=np.int32)
            else:
                ids = rng.integers(0, V, size=Bp).astype(np.int32)
            out = ost.step(ids, n_total - len(ost.emitted))
            B.la_jacobi_accept(eng.kv, k, B.to_device(ids), state, emitted, n_total)
            st = B.read_state(state)
            assert st.last_emitted == len(out) and st.n_emitted == len(ost.emitted)
            assert st.steps == ost.iterations and st.matched_steps == ost.blocks
            assert (st.last_m == ost.last_iterations) and B.la_kv_get_len(eng.kv) == ost.t
            passes += 1
        assert np.array_equal(emitted.cpu().numpy(), np.asarray(ost.emitted))
        B.la_jacobi_accept(eng.kv, k, B.to_device(ids), state, emitted, n_total)   # budget spent: a no-op
        st = B.read_state(state)
        assert st.last_emitted == 0 and st.n_emitted == n_total and st.steps == ost.iterations
    finally:
        eng.close()


def test_jacobi_tiny_decoder_equals_oracle_jacobi_and_sequential():
    """End to end on the fp32 path: the GPU's Jacobi stream, its pass count and its committed
    cache against the oracle's Jacobi loop (whose stream is pinned to greedy decoding)."""
    shape = synth.SHAPES["tiny_f32"]
    om = oracle_model(shape, seed=0)
    prompt = synth.uniform_prompt(shape.vocab, 32, 0)
    want, lgs, _ = otf.greedy_sequential(om, prompt, 32, return_logits=True)
    t1, t2 = otf.top2_margin(lgs)
    assert np.all(t1 - t2 > 1e-6)
    owant, ost, okv = ojc.greedy_jacobi(om, prompt, 32, 6, Bp=8)
    assert np.array_equal(owant, want)
    eng = gpu_engine(shape, 32 + 32 + 16, seed=0)
    try:
        seq, _ = eng.generate(prompt, 32, 0, 1, 0)
        got, st = eng.generate_jacobi(prompt, 32, 6, Bp=8)
        assert np.array_equal(got, seq)
        first_bad = next((i for i in range(32) if got[i] != want[i]), None)
        if first_bad is None:
            assert st["passes"] == ost.iterations and st["blocks"] == ost.blocks
            for l in range(shape.n_layers):
                k, v = eng.read_kv(l, 0, st["L"])
                assert np.max(np.abs(k - okv.K[l, :st["L"]])) <= 1e-4 * np.max(np.abs(okv.K[l, :st["L"]]))
                assert np.max(np.abs(v - okv.V[l, :st["L"]])) <= 1e-4 * np.max(np.abs(okv.V[l, :st["L"]]))
        else:
            assert t1[first_bad] - lgs[first_bad, got[first_bad]] <= MARGIN
        print(f"jacobi k=6: {st['passes']} passes for 32 tokens ({st['tokens_per_pass']:.2f} tokens per pass)")
    finally:
        eng.close()


@pytest.mark.parametrize("name,k", [("small_bf16", 8), ("small64_bf16", 5)])
def test_jacobi_on_the_matrix_core_path(name, k):
    """bf16 shapes: Jacobi == sequential on the same engine (a pass's rows do not depend on the
    block they rode in), and on a closed-form successor model exactly k passes per block."""
    from paper_2602_16760_amd.engine import Engine
    from test_gpu_parity import _orbit_model
    shape = synth.SHAPES[name]
    base = synth.uniform_prompt(shape.vocab, 12, 3)
    prompt = np.concatenate([base, base, base[:5]])
    eng = gpu_engine(shape, 256, seed=2)
    try:
        seq, _ = eng.generate(prompt, 40, 0, 1, 0)
        got, st = eng.generate_jacobi(prompt, 40, k)
        same = got == seq
        if not same.all():   # they may part only where the oracle's margin is thin
            om = oracle_model(shape, seed=2)
            i = int(np.argmin(same))
            _, lg = otf.causal_forward(om, np.concatenate([prompt, seq])[:len(prompt) + i])
            t1, t2 = otf.top2_margin(lg[-1:])
            assert t1[0] - t2[0] <= MARGIN
        assert st["passes"] <= 40 + st["blocks"]
        print(f"{name} jacobi k={k}: {st['passes']} passes for 40 tokens ({st['tokens_per_pass']:.2f} per pass)")
    finally:
        eng.close()
    period = 5
    perm, layer, head = _orbit_model(shape, period, 4)
    eng = Engine(shape, 256, layer, head)
    try:
        p = [3 * period + 2]
        for _ in range(6):
            p.append(int(perm[p[-1]]))
        got, st = eng.generate_jacobi(np.asarray(p, dtype=np.int32), 4 * k, k)
        expect = []
        cur = p[-1]
        for _ in range(4 * k):
            cur = int(perm[cur])
            expect.append(cur)
        assert list(got) == expect
        assert st["passes"] == 4 * k and st["blocks"] == 4      # one token settles per pass: Section 4.2's poor convergence
    finally:
        eng.close()
