"""CPU oracle for one mixed-batch serving iteration of a decoder-only transformer.

TEST INFRASTRUCTURE ONLY.  This tree is a plain, slow, obviously-correct numpy
statement of what the serving step computes (PolyServe, Sec. 2.1 "LLM Inference
Workflow": RMS-normalised attention module with Softmax(QK^T/sqrt(d))V over all
previous tokens, O-projection, gated feed-forward network, residual connections;
Sec. 2.4: a chunk of prefill tokens batched with all running decode tokens).
It exists so that the GPU kernels have something independent to be compared
against.  It shares no code with the HIP library or its Python binding and
imports neither; only tests, the smoke entry and the benchmark's CPU-baseline
leg may import it.

Modules
  bf16      bfloat16 <-> float32 bit conversions (round-to-nearest-even).
  indices   integer side of a step: cu_seqlens / positions / slot mapping,
            and the seeded page allocator.
  layer     floating-point side: RMSNorm, RoPE, paged KV append, causal paged
            attention, SwiGLU feed-forward, one layer and a stack of layers.

Pins (tests/test_oracle_*.py): brute-force dense fp64 attention, torch's
scaled_dot_product_attention / rms_norm / silu as library special cases,
chunked-vs-one-shot prefill invariance, decode with one key returns V exactly,
page-permutation invariance, RoPE isometry and relative-position property,
GQA-vs-expanded-MHA, closed forms for every index array, and an independently
written shuffle for the allocator.  No function here is "parity unpinned".
"""
