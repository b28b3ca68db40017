"""CPU oracle for the split (two-stage) backward pass of a LLaMa-like decoder stage.

TEST INFRASTRUCTURE ONLY.  This package is the slow, plain definition that the HIP library is
checked against.  It is imported by the tests, by the smoke check and by the benchmark's CPU
baseline leg, never by the product path, and it shares no code with the HIP kernels.

What it follows: the paper's Section 3.1 (backward-p1 = gradient w.r.t. the previous layer's
output, backward-p2 = gradient w.r.t. the layer's parameters, p2 deferrable), Section 3.2 (every
module has forward and backward-p1, parametrised modules also backward-p2; p2 right after p1
reproduces ordinary backpropagation; micro-batches may be concatenated over the batch dimension
so that p2 is called once) and Section 4.2 (linear layers keep input activation and output
derivative until p2; functional operations release their activations in p1).  The paper lists the
Transformer-7b ingredients (rotary embedding, SwiGLU MLP, RMSNorm, no linear bias) without
formulas; the formulas here are the standard definitions of those ingredients.

Because 2BP only re-orders an exact computation, the oracle is the plain analytic gradient,
evaluated in fp64 (an fp32 switch exists) with numpy; `matmul` is the only library primitive used
as a step.  Pins (tests marked "not gpu"): central finite differences, equality of split and
monolithic backward, accumulated == concatenated weight gradients, closed-form linear-layer
gradients, library routines (rms_norm, silu, scaled_dot_product_attention, autograd) on special
cases, and algebraic invariants of each operation.  Every function is pinned.
"""
from .ops import (  # noqa: F401
    linear_fwd, linear_p1, linear_p2,
    rmsnorm_fwd, rmsnorm_p1, rmsnorm_p2,
    swiglu_fwd, swiglu_p1,
    rope_fwd, rope_p1,
    softmax_fwd, softmax_p1,
    attention_fwd, attention_p1,
)
from .stage import OracleStage  # noqa: F401
from .monolithic import monolithic_backward  # noqa: F401
