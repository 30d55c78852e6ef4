"""CPU oracle for the entropy-routed stitched decoding hot path.

TEST INFRASTRUCTURE ONLY.  This package is a plain, slow, fp64 implementation
of what the HIP library computes, written from the paper's definitions (and,
for the decoder forward pass the paper leaves to "a full forward pass", from
the public definition of the Qwen2-style decoder layer).  It may be imported by
``tests/``, by ``__graft_entry__.smoke()`` and by the ``cpu_baseline`` leg of
``bench.py`` and by nothing else; it imports nothing from the HIP package and
shares no code, tables or constants with it.

Modules
  router   normalised token entropy (Eq. 1), switching rule (Eq. 2)
  decoder  RMSNorm, rotary embedding, grouped-query attention over a KV cache,
           SwiGLU MLP, LM head; one forward invocation over a span of tokens
  stitch   the inference loop of Algorithm 1 with two KV caches (and its R-Stitch+ branch)
  router_plus  the learned router of R-Stitch+ (six residual FFN blocks, LayerNorm, two outputs)

Parity status: every function here is pinned by ``tests/test_oracle_*.py``
(closed forms, brute force, an independent library implementation of the same
decoder).  Nothing is "parity unpinned".
"""
