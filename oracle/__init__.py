"""CPU oracle for the virtual-node training step (VirtualFlow, arxiv 2009.09523).

TEST INFRASTRUCTURE ONLY.  Nothing on the product path may import this package:
only the tests, the smoke check and the benchmark's cpu_baseline leg use it.  It
shares no code with the HIP library and never calls it.

It is the plain definition of what one step computes (Section 3.2, steps 1-5,
with the weights of Section 5.2), written in NumPy float64:

  1. split the batch of B rows into V contiguous virtual nodes of sizes b_i;
  2. for every node alone: forward pass in training mode (BatchNorm statistics
     over that node's rows only), mean loss L_i, gradient g_i of L_i;
  3. G = sum_i (b_i/B) g_i and L = sum_i (b_i/B) L_i   (Section 5.2);
  4. one optimizer update with G                        (Section 3.2, step 5).

bf16 workloads are defined as "bf16 weights and activations, fp32 accumulation,
fp32 master weights", their contractions being bf16 products: the oracle rounds
the fp32 master parameters to bf16 (round-to-nearest-even) before the passes and
rounds every operand of a contraction (Linear, convolution, attention product;
forward and backward) to bf16 where it is produced.  Everything else -- what a
contraction puts out included -- is float64.  Which tensors this rule
rounds is fixed by this build's reading of that phrase, not by the paper
("parity unpinned": the float64 pins run without any rounding); a workload whose
dtype is not bf16 is evaluated without it, which is how tests obtain the
weights-only-rounded evaluation of the same step.

Pins (tests/test_oracle_*.py): the 6+2 worked example of Section 5.2 with its
unweighted negative control; partition-invariance of G without BatchNorm;
V = 1 fallback; central finite differences of the combined loss for every
layer type; torch float64 autograd run per node slice; closed forms for the
loss (ln N for uniform logits) and for both optimizers.

Readings of the paper that nothing in it pins ("parity unpinned": the HIP path
and this oracle simply agree on them): SGD-momentum form and learning rates,
Adam epsilon, BatchNorm/LayerNorm epsilon, masked-position recipe of the
encoder workload, absence of dropout.
"""
from .partition import partition, node_of_sample
from .numerics import round_to_bf16
from .optim import sgdm_update, adam_update
from .step import oracle_step, node_loss_and_grads, unflatten, layout

__all__ = ["partition", "node_of_sample", "round_to_bf16", "sgdm_update", "adam_update",
           "oracle_step", "node_loss_and_grads", "unflatten", "layout"]
