#!/usr/bin/env python3
"""Benchmark of the lookahead verification step on one MI355X.

    python bench.py --gpus 1 --steps K --warmup W

Workload (BASELINE config 2, the one the metric is quoted on): Mistral-7B-shaped cloud
share, 30 layers, bf16, random N(0, 0.02) weights, KV cache pre-filled to 512 positions with
N(0, 1) activations, 32-row lookahead block (W=5, N=4, G=5: 31 rows + 1 pad).  One step is
the whole hot path on one block: embedding gather of the block's tokens, the 30-layer stack
under the lookahead mask, final norm + unembedding + greedy arg-max at every row, n-gram
acceptance with KV commit and construction of the next block -- all enqueued without a host
synchronisation; the state lives on the device.  Inputs are resident in HBM before timing.

Prints one JSON line.  `value` = block rows verified per second.  `roofline` is measured
with HIP events around the dominant kernel's launches during the timed steps;
`cpu_baseline` times the float64 oracle on a bounded sample of the same workload.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time
from concurrent.futures import ThreadPoolExecutor

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

W_LA, N_LA, G_LA, BP = 5, 4, 5, 32
L0 = 512
N_LAYERS = 30
PEAK_HBM_GBPS = 8000.0


def log(*a):
    print("[bench]", *a, file=sys.stderr, flush=True)


def build_engine(shape, max_len, seed=0):
    import torch
    import synth
    from paper_2602_16760_amd.engine import Engine

    t0 = time.time()
    head = synth.head_weights(shape, seed, unit_gains=True)
    eng = Engine(shape, max_len, None, head)
    del head
    # generate layers on host threads (numpy releases the GIL), upload and pack one at a time
    with ThreadPoolExecutor(max_workers=min(8, os.cpu_count() or 8)) as ex:
        futs = [ex.submit(synth.layer_weights, shape, l, seed, True) for l in range(shape.n_layers)]
        for l, f in enumerate(futs):
            eng.set_layer(l, f.result())
            futs[l] = None
            if l % 5 == 4:
                log(f"layer {l + 1}/{shape.n_layers} uploaded ({time.time() - t0:.0f} s)")
    for l in range(shape.n_layers):
        k, v = synth.kv_fill(shape, l, L0, seed)
        eng.fill_kv(l, k, v)
    torch.cuda.synchronize()
    log(f"model + cache resident after {time.time() - t0:.0f} s")
    return eng


def algorithmic_bytes(shape, n_layers, L, Bp):
    """Bytes one step must move: every weight once, every live KV row once, block KV written once."""
    d, F, qd, kvd = shape.d_model, shape.d_ffn, shape.q_dim, shape.kv_dim
    per_layer = 2 * (d * (qd + 2 * kvd) + qd * d + 2 * d * F + F * d)
    kv_read = 2 * 2 * L * kvd
    kv_write = 2 * 2 * Bp * kvd
    unembed = 2 * d * shape.vocab
    return n_layers * (per_layer + kv_read + kv_write) + unembed


def cpu_baseline(shape):
    """The oracle as it stands on the host cores: one layer of the 30, same block and cache."""
    import synth
    from oracle import lookahead as ola
    from oracle import transformer as otf

    sh1 = shape.with_layers(1)
    w = synth.layer_weights(sh1, 0, 0, True)
    om = otf.Model(sh1, lambda l: w, None, cache=True)
    om.layer(0)  # widen outside the timed region: it stands in for weights resident in memory
    kv = otf.KVCache(sh1, L0 + BP, 1)
    k, v = synth.kv_fill(sh1, 0, L0, 0)
    kv.fill(0, k, v)
    kv.L = L0
    _, pos, vis = ola.build_block(0, L0, [[0] * W_LA for _ in range(N_LA - 1)], [(0,) * (N_LA - 1)] * G_LA,
                                  W_LA, N_LA, G_LA, BP)
    x = synth.hidden_block(sh1, BP, 0)
    # about ten seconds of oracle work: one warm-up pass, then as many passes as fit (at most 400)
    otf.forward_block(om, kv, x, pos, vis)
    reps, t0 = 0, time.time()
    while reps < 400 and (reps < 3 or time.time() - t0 < 10.0):
        otf.forward_block(om, kv, x, pos, vis)
        reps += 1
    dt = (time.time() - t0) / reps
    rows = ola.block_rows(W_LA, N_LA, G_LA)
    return {
        "value": rows / (dt * N_LAYERS),
        "unit": "tok/s",
        "cores": int(os.environ.get("OMP_NUM_THREADS", os.cpu_count() or 1)),
        "kind": "oracle",
        "sample": f"1 of {N_LAYERS} layers (float64 numpy, {BP}-row block, L={L0}), {reps} repetitions, "
                  f"{dt:.2f} s per layer, step time extrapolated x{N_LAYERS}; unembedding not included",
    }


def measured_traffic():
    """HBM bytes per launch of the dominant kernel from the committed rocprofv3 --pmc summary
    (FETCH_SIZE + WRITE_SIZE, scaled by a copy kernel of known size), or None."""
    path = os.path.join(ROOT, "profiles", "layer_stack_config2_pmc.txt")
    try:
        with open(path) as f:
            for line in f:
                if line.startswith("traffic_bytes_per_launch:"):
                    return int(float(line.split(":", 1)[1].split()[0]))
    except OSError:
        pass
    return None


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--layers", type=int, default=N_LAYERS, help=argparse.SUPPRESS)
    ap.add_argument("--calib-copy", action="store_true",
                    help="also launch a 1 GiB copy kernel (calib_copy) before the timed steps: a dispatch of known "
                         "traffic for scaling rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE readings")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (no collectives, no sharding); use --gpus 1", file=sys.stderr)
        sys.exit(2)

    import torch
    import synth
    from paper_2602_16760_amd import binding as B

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(1)
    n_layers = args.layers
    shape = synth.SHAPES["mistral7b"].with_layers(n_layers)
    rows = 1 + (W_LA + G_LA) * (N_LA - 1)
    total_steps = args.warmup + args.steps + 8
    max_len = L0 + total_steps * N_LA + BP + 64
    eng = build_engine(shape, max_len)

    # controller: prompt of L0+1 synthetic "code-like" tokens seeds the pool; the cache rows
    # 0..L0-1 are the N(0,1) fill, so nothing is prefilled through the model
    prompt = synth.markov_prompt(shape.vocab, L0 + 1, 0.30, 0)
    eng.start(prompt, W_LA, N_LA, G_LA, BP, seed_pool=True, prefill=False)
    budget = total_steps * N_LA + 16
    emitted = torch.zeros(budget, dtype=torch.int32, device="cuda")

    for _ in range(args.warmup):
        eng.step(emitted, budget)
    torch.cuda.synchronize()
    if args.calib_copy:
        src = torch.ones(1 << 28, dtype=torch.int32, device="cuda")   # 1 GiB read + 1 GiB written
        dst = torch.empty_like(src)
        for _ in range(2):
            B.la_profile_copy(dst, src)
        torch.cuda.synchronize()
        del src, dst
    st0 = B.read_state(eng.state)

    dominant = "layer_stack"   # the persistent kernel that runs all layers of the step
    B.la_profile_select(dominant)
    B.la_profile_enable(True)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        eng.step(emitted, budget)
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    B.la_profile_enable(False)
    prof = B.la_profile_read()
    B.la_profile_select(None)
    st1 = B.read_state(eng.state)
    ms_per_step = dt * 1e3 / args.steps

    # attribution pass (not timed): every kernel bracketed
    B.la_profile_enable(True)
    for _ in range(3):
        eng.step(emitted, budget)
    torch.cuda.synchronize()
    B.la_profile_enable(False)
    allk = B.la_profile_read()
    per_step = {k: round(v[1] / 3.0, 4) for k, v in sorted(allk.items(), key=lambda kv: -kv[1][1])}
    log("per-step kernel ms (event-bracketed pass):", json.dumps(per_step))

    # the same step with a one-row block (sequential decoding): the method's premise is that a
    # 32-row verify step costs about what a one-token step costs (Section 4.2)
    L_seq = int(st1.L) + 3 * N_LA
    B.la_kv_set_len(eng.kv, L_seq)
    eng.start(np.concatenate([prompt, prompt[: L_seq + 1 - len(prompt)]])[: L_seq + 1], 0, 1, 0, 1, seed_pool=False, prefill=False)
    seq_emitted = torch.zeros(64, dtype=torch.int32, device="cuda")
    for _ in range(3):
        eng.step(seq_emitted, 64)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(20):
        eng.step(seq_emitted, 64)
    torch.cuda.synchronize()
    seq_ms = (time.perf_counter() - t0) * 1e3 / 20

    L_mid = (st0.L + st1.L) / 2.0
    step_bytes = algorithmic_bytes(shape, n_layers, L_mid, BP)
    gbps = step_bytes / (ms_per_step * 1e-3) / 1e9
    launches, total_ms = prof.get(dominant, (0, 0.0))
    # per launch: every layer's weights once, every live KV row once, the block's KV written once
    dom_bytes = int(algorithmic_bytes(shape, n_layers, L_mid, BP) - 2 * shape.d_model * shape.vocab)
    dom_ms = total_ms / max(launches, 1)
    dom_gbps = dom_bytes / (dom_ms * 1e-3) / 1e9 if dom_ms > 0 else 0.0

    out = {
        "metric": "lookahead-step ms + verified tok/s + HBM GB/s % peak, Mistral-7B-shape 30 layers",
        "value": round(rows / (ms_per_step * 1e-3), 1),
        "unit": "verified tok/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 4),
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "bf16",
        "data": "synthetic",
        "config": {
            "workload": f"Mistral-7B-shape cloud share, {n_layers} layers, KV prefilled to {L0}, "
                        f"{BP}-row lookahead block (W={W_LA}, N={N_LA}, G={G_LA}: {rows} rows + pad), batch 1, "
                        "plus embedding gather, unembedding (vocab 32768) + arg-max, n-gram accept + KV commit",
            "block_rows": BP, "kv_len_start": int(st0.L), "kv_len_end": int(st1.L),
            "arithmetic": "bf16 weights and KV cache; the weight GEMMs multiply the weights as f16 (the conversion is exact) "
                          "with f16 activations and f32 accumulation; attention on bf16 MFMA; residual stream f32",
        },
        "step_hbm_gbps": round(gbps, 1),
        "step_hbm_frac_peak": round(gbps / PEAK_HBM_GBPS, 4),
        "step_algorithmic_bytes": int(step_bytes),
        "accepted_tok_per_step": round((st1.n_emitted - st0.n_emitted) / max(st1.steps - st0.steps, 1), 3),
        "emitted_tok_per_s": round((st1.n_emitted - st0.n_emitted) / dt, 1),
        "kernel_ms_per_step": per_step,
        "one_row_step_ms": round(seq_ms, 4),
        "block_to_one_row_latency_ratio": round(ms_per_step / seq_ms, 3),
        "roofline": {
            "bound": "hbm", "kernel": dominant, "achieved": round(dom_gbps, 1), "peak": PEAK_HBM_GBPS, "unit": "GB/s",
            "frac": round(dom_gbps / PEAK_HBM_GBPS, 4), "traffic": measured_traffic(),
            "bytes_per_launch": dom_bytes, "launches": launches, "avg_launch_ms": round(dom_ms, 5),
        },
    }
    if not args.no_cpu_baseline:
        log("timing the float64 oracle on one layer (host cores) ...")
        out["cpu_baseline"] = cpu_baseline(shape)
    eng.close()
    print(json.dumps(out), flush=True)


if __name__ == "__main__":
    main()
