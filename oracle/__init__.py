"""CPU oracle for the per-layer MoE prefill block (router, top-k, grouping,
grouped SwiGLU expert FFN, weighted combine).

TEST INFRASTRUCTURE ONLY.  Nothing in the product package may import this
directory: only tests/, __graft_entry__.smoke() and bench.py's cpu_baseline leg
use it.  It shares no code, table or constant generator with the HIP path.

Modules
  codecs      software bf16 / OCP e4m3 encoders and decoders (numpy)
  moe_oracle  the block in fp64 (numpy), written from the definition in
              Sec. 2.3 of the paper (E experts, each a two-layer MLP; a router
              sends every token to its top-k experts and sums their outputs)
  brute       pure-Python loops for tiny inputs, and a loader for the plain C
              triple-loop twin (brute_moe.c) used at the tiny-layer size

Parity pins (tests/test_oracle_*.py): brute-force loops, closed forms
(softmax over the selected logits, dense SwiGLU for E=1,k=1), invariants
(counts sum to T*k, bijective permutation, weights sum to 1, identical experts
collapse to one expert), scaling laws, an enumerated e4m3 table and torch's CPU
casts as an independent codec; down_project (the second expert GEMM on its own)
against a hand-worked case, plain loops and the layer's own y.  No function here
is "parity unpinned".
"""
