"""CPU oracle for the lookahead-decoding verification step (fp64, numpy).

TEST INFRASTRUCTURE ONLY.  This package is the slow, plain definition that the
HIP path is checked against.  Only tests/, __graft_entry__.smoke() and the
cpu_baseline leg of bench.py may import it.  It shares no code with the HIP
path and imports nothing from it; both read the same seeded inputs from the
`synth` package.

Contents
  transformer.py  Mistral-family decoder layer stack in float64: RMSNorm, RoPE,
                  grouped-query attention over a KV cache with an explicit
                  per-row visibility set, SwiGLU MLP, final norm + unembedding
                  + greedy argmax.  Three entry points: a dense full-sequence
                  causal pass (the textbook definition), one-token-at-a-time
                  greedy decoding (the paper's sequential baseline, Section 4.1)
                  and a block forward under an arbitrary visibility mask
                  (Sections 3.3 and 4.4).
  lookahead.py    Integer logic of lookahead decoding (Section 4.3): block
                  layout, visibility masks, n-gram pool, verification,
                  acceptance, KV commit list, window update.

Pins (tests/test_oracle_*.py, all CPU): greedy lookahead output equals
sequential greedy output token for token (the paper's Section 6.5 invariant);
every block row equals the dense causal pass on that row's own pseudo-sequence;
the plain causal mask the paper prints in Section 4.4 reproduces the dense
causal pass and a cache-relative mask does not; closed forms for RMSNorm, RoPE,
softmax and SiLU; an independent torch float64 implementation of one layer;
brute-force argmax with ties; integer bounds 1 <= emitted <= N per step.

Parity unpinned: acceptance *rates* against the paper's Section 6.4 tables
(they depend on trained weights and the paper's prompts, which are absent).
"""
