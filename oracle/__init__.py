"""CPU oracle for the RMM linear layer (test infrastructure, not product code).

Plain, slow, fp64 numpy statement of what the randomized-matrix-multiplication
linear layer computes (paper: Section 2.1, Eq. 1-5, Algorithm 1; Section 2.3,
Lemmas 2.1-2.2 and the B=2 worked example).  It exists only so that tests, the
smoke check and the bench's cpu_baseline leg have something independent of the
HIP kernels to compare with.  Nothing in the product package imports it, and it
imports nothing from the product package.

Modules
-------
philox    Philox-4x32-10 counter-based generator (integer only).
sketch    counter -> element map of the virtual N x k sketch S (Gaussian, Rademacher).
rmm       Algorithm 1 forward / backward on an explicitly materialised S, plus the
          exact gradients of Eq. 2-3 the estimator targets.
variance  closed-form variances of the estimator and the monitors of Section 2.3.

Pins (tests/test_oracle_*.py, all CPU-only): published Philox known-answer
vectors, brute-force triple loops, Monte-Carlo unbiasedness, closed-form
variances on correlated inputs, sample moments, the paper's worked example.
"""
from . import philox, sketch, rmm, variance  # noqa: F401
