"""fp64 CPU oracle for the activation-reuse training path (TEST INFRASTRUCTURE ONLY).

This package is the slow, plain definition of what the HIP library computes.  It is
test infrastructure: only the test-suite, the smoke check and the CPU-baseline leg
of the benchmark may import it.  It shares no code with the HIP path and imports
nothing from it; every function works on numpy float64 arrays (integer / byte
arrays for the gather) and uses library matmuls as single steps with no blocking,
fusion or reordering beyond what the definitions state.

Paper basis (Alchemist, arXiv 2503.01066): Section 1 and Section 2.5.1 state that
the activations produced while serving a prompt are the same tensors the training
forward pass would produce, so back-propagation may start from them; Section 4.1
restricts the recording to the prefill phase; Sections 4.2 and 4.3.2 run the
backward pass layer by layer from the output layer to the input layer; Section 5
names the cross-entropy loss on the prefill output; Section 6 names the model
family (Llama-3.1-8B, Mistral, Phi-4: pre-norm decoders with RMSNorm, rotary
embeddings, grouped-query attention and a SwiGLU MLP).  The paper prints no
formula; the layer function below is that model family's standard definition.

Modules:
  gather  -- selection-mask gather / pack of activation rows (exact, byte-wise)
  layer   -- decoder-layer forward, and backward from a saved record (reuse) or
             from a recomputed forward (recompute)
  stack   -- L-layer stack with final norm, LM head and cross-entropy loss
  lora    -- the layer with low-rank adapters on its projections (Section 3 A1, Section 6: rank 8)
  prefix  -- sequences that share a prefix (responses on the saved KV cache of their prompt, Section 4.1)
             and the DPO loss on them (Section 6)
Every function is pinned by tests/test_oracle_*.py (finite differences, the
reuse == recompute invariant, brute-force gather, closed forms, special cases).
"""
from .gather import gather_pack
from .layer import (LayerShape, layer_forward, layer_backward_reuse,
                    layer_backward_recompute, complete_record, attention_lse, RECORD_KEYS, WEIGHT_KEYS)
from .stack import stack_forward, stack_backward_reuse, stack_backward_recompute
