"""CPU oracle for Parallel Restarted SGD -- TEST INFRASTRUCTURE, not a product path.

A plain, slow, obviously-correct numpy/float64 implementation of what the HIP
path computes, written from the paper (Algorithm 1, eq. 2-6; Algorithms 2 and 3).
It shares no code with the HIP library and never imports it.  Only the tests,
the smoke check and the benchmark's CPU-baseline leg may import this package;
the product path must never route through it.

Pins (tests/test_oracle_*.py, all run without a GPU):
  index sampler     Philox4x32-10 known-answer vectors; uniformity
  gradients         finite differences; torch.autograd (float64); closed forms
  Algorithm 1       I=1 == mini-batch SGD with the averaged gradient; N=1 == SGD;
                    eq. (5) mean recursion; eq. (6) restart identity; replicas
                    equal after every restart
  Algorithms 2, 3   reduce to Algorithm 1 for constant (gamma, K) / equal I_i; Algorithm 2 with
                    epochs of different lengths and rates against a loop written out in the
                    test and against the closed form of a one-row least-squares problem;
                    Theorem 2's K^s against its exact integer definition
  momentum          mu = 0 is Algorithm 1; geometric closed form under a constant gradient;
                    N = 1 against an independently written heavy-ball loop; I = 1 with
                    averaged buffers == momentum SGD on the averaged gradient; mean recursion
  bf16 rounding     torch's float32 -> bfloat16 conversion (NaN and infinity included)
  bf16 operand mode nets with hidden layers against an emulation built from torch.bfloat16 casts;
                    a hand-sized net whose expected values are exact binary fractions and which
                    fails when any single rounding point is left out

Parity unpinned: the long-horizon (thousands of non-convex steps) trajectory has
no reference other than this oracle itself.
"""
from .philox import philox4x32_10, sample_rows  # noqa: F401
from .models import (  # noqa: F401
    round_bf16,
    lsq_loss_grad,
    mlp_loss_grad,
    mlp_unflatten,
    loss_grad,
)
from .prsgd import (  # noqa: F401
    run_prsgd,
    momentum_step,
    run_prsgd_literal,
    run_time_varying,
    run_heterogeneous,
    time_varying_schedule,
    node_average,
)
