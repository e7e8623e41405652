"""CPU oracle for the SPB worker step.  TEST INFRASTRUCTURE, not product code.

A plain, slow float64 statement of what one worker computes under Structured
Partial Backpropagation (Sec. 2 of the paper): the full forward pass to the
loss, then ordinary backpropagation over the top k units only.  Only the test
suite, the smoke check and the benchmark's reported CPU baseline may import
it; the HIP path never does, and shares no code with it.

Pins (tests/test_oracle_*.py): finite differences on tiny nets, closed forms of
the softmax cross-entropy, brute-force loops for the matrix products, the
suffix invariants of Sec. 1-2 (depth L equals full backprop, depth 0 yields
nothing, gradients above the cut do not depend on the cut), and torch's CPU
autograd as a third opinion at full size.
"""
from .bf16 import round_to_bf16  # noqa: F401
from .spb import spb_step, build_units, identity  # noqa: F401
from .aggregate import aggregate_update, worker_depths, contributors  # noqa: F401
from . import jigsaw  # noqa: F401
