"""CPU oracle for one GPU's share of a sharded data-parallel transformer training step.

TEST INFRASTRUCTURE ONLY.  This package is the slow, plain, fp64 statement of what the
HIP library computes.  Only the test-suite, the smoke check and the benchmark's
CPU-baseline leg may import it; the product path never does.  It shares no code with
the HIP path and imports nothing from it.

What it states (Cephalo, arXiv 2411.01075):
  * Sec. 3.1 "Compute Partitioning", Eq. 1: a GPU's local gradient over its batch share
    b_i is scaled so that the average over GPUs equals the plain 1/B mean.
  * Sec. 3.1 "Training State Partitioning": the GPU owns a contiguous slice of ratio r_i
    of the flat parameter / gradient / Adam-moment buffers of an FSDP unit and applies
    the optimizer to that slice only.
  * Sec. 3.2: the share is processed as l micro-batches of size m (b = l * m) whose
    gradients are accumulated; with layered accumulation all micro-batches pass through
    a layer before the next layer.
  * Sec. 2.1 / Sec. 3.3 "Memory Utilization Model": a transformer layer (self-attention +
    feed-forward) trained with Adam, 16 bytes of training state per parameter.

  * Sec. 3.3 performance models (oracle.perfmodel) and Sec. 3.4 optimizer (oracle.plan: the
    optimization problem by exhaustive search, the state partition as a linear programme).

Because the method reproduces standard training exactly (Eq. 1 is an identity; sharding
only moves where an element's update runs), every function here is the textbook
definition written out, not a re-derivation of any kernel.

Pins (tests/test_oracle_*.py): finite differences and torch autograd for every gradient,
pure-Python triple loops on tiny shapes, closed forms for LayerNorm / softmax / GELU /
first-step Adam, torch.optim.Adam for the unsharded update, the micro-batch-sum and
shard-partition invariants, and Eq. 1 with uneven shares.  The whole-stack loss value
(oracle.stack) has no printed value in the paper to compare with: its pins are finite
differences and autograd only.  oracle.llama (the Llama-style layer: RMSNorm, rotary embedding, gated SiLU feed-forward, no biases; and a stack of
them with a token embedding, a final RMSNorm and a head of its own) is pinned
by tests/test_oracle_llama.py: closed forms, rotation invariants, finite differences and an independent torch
implementation under autograd.  oracle.perfmodel is pinned by closed forms of the line fit and
by the latencies and memory the paper plots (tests/golden/); oracle.plan is the definition
itself (every assignment enumerated), used on tiny clusters only.
"""
