"""CPU oracle for the local-update step.  TEST INFRASTRUCTURE ONLY.

Plain numpy, float64 by default, written from the paper's definition of the method (section 3,
appendices A-B).  Only tests, the smoke check and the bench's CPU-baseline leg may import it; the
product path never does, and it shares no code with the HIP kernels.

Pinned (tests/test_oracle_*.py) by finite differences per head with the window input frozen,
the exact-zero gradient across truncation boundaries, the reductions to ordinary backprop
(one head with a full window; last block of the greedy scheme), the deep-supervision sum,
closed forms (zero head => loss = ln C), brute-force loops for convolution / attention /
optimizers on tiny shapes, and independent library routines (torch CPU autograd) for each
primitive and for a whole decoder layer.  The paper prints no numeric example of a step, so the
end-to-end values themselves are pinned only through those properties.  The running statistics of
batch normalisation (a convention the paper leaves open) are pinned by torch's BatchNorm2d on CPU, a
closed form on a repeated batch, and the identity "normalising with the batch's own statistics repeats
batch mode" on a whole model.
"""
from .ops import BatchNormRunning
from .local import (eval_loss, local_gradients, local_step, block_gradients, new_state,
                    forward_all, optimizer_update, layer_gradient_cosines, new_pipeline, pipelined_step)

__all__ = ["eval_loss", "local_gradients", "local_step", "block_gradients", "new_state",
           "forward_all", "optimizer_update", "layer_gradient_cosines", "new_pipeline", "pipelined_step",
           "BatchNormRunning"]
