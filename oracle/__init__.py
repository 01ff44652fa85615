"""CPU oracle for the per-GPU hot path of PTD-P training (arXiv 2104.04473).

TEST INFRASTRUCTURE ONLY.  This package is the slow, plain, fp64 definition of
what the HIP library computes.  It is imported by ``tests/``, by
``__graft_entry__.smoke()`` and by the ``cpu_baseline`` leg of ``bench.py`` and
by nothing else; the product package never imports it and it never imports the
product package.  It shares no code, tables or constants generators with the
HIP path: both sides restate the same definitions independently.

Modules
-------
dropout_hash  counter-based dropout mask (integer, bit-exact on both sides)
gpt_layer     forward / backward of one tensor-parallel shard of a GPT layer (causal or general mask)
flops         the paper's closed forms (eq. 1, eq. 2, eq. 3, appendix, 8TP/nX)
schedule      1F1B / interleaved 1F1B order of one device + p-device simulator
recompute     activation recomputation: memory model of section 3.5, backward from checkpoints
lm_stage      first / last stage extras: embeddings, final LayerNorm, logit layer, loss

Parity status: every function here is pinned by ``tests/test_oracle_*.py``
(finite differences, an independent autograd derivation, closed forms,
invariants, degenerate cases, brute-force simulation).  Nothing is
"parity unpinned"; note that the paper prints no numeric layer example, so
absolute activation values are pinned through mathematics, not through a
table of the paper.
"""
