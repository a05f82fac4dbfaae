"""CPU oracle: a plain, slow, obviously-correct implementation of the speculative
draft/verify path.

TEST INFRASTRUCTURE ONLY.  Nothing in the product (the HIP library and its Python
binding) may import or call this package; only ``tests/``, the smoke check and the
``cpu_baseline`` leg of the benchmark do.  It shares no code with the HIP path.

Modules
  model.py   decoder forward (RMSNorm, RoPE, GQA attention with a KV cache, top-2 MoE or
             dense SwiGLU, LM head) in float64 NumPy
  spec.py    plain decoding, greedy speculative decoding, stochastic speculative sampling,
             the accept/reject rule on given logits, the expected-length law
  philox.py  Philox4x32-10 and the uniform stream layout
  counts.py  parameter / byte / FLOP counts of a model shape, memory model of the planner
"""
