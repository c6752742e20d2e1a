"""CPU oracle for one GPU's section compute (TEST INFRASTRUCTURE ONLY).

This package is the slow, plain, fp64 definition of what the HIP library
computes: decoder / encoder section forward and backward on packed
variable-length tokens, and the temperature-softmax KL distillation loss that
joins a forward-only teacher to a forward+backward student (paper Sec. 2.2,
Sec. 3.1).  It depends on numpy (+ scipy.special.erf) only, shares no code
with the HIP path and must never be imported by the product package; only the
tests, the smoke check and the CPU-baseline leg of the benchmark call it.

Every tensor is a float64 ndarray, row-major, packed `[N, features]` with
`cu_seqlens[B+1]` giving sequence boundaries.  `rnd` arguments are the
"materialisation rounding": identity (pure fp64, used by the pins) or
round-to-nearest-even to bf16 (used for parity with the bf16 HIP path, which
stores exactly those tensors in bf16 while accumulating in fp32); `rnd_res`
is the same for the forward residual stream, which the bf16 HIP path keeps in
fp32 (round_f32).

Parity status: the paper prints no worked numeric example of this path, so the
oracle is pinned by closed forms, invariants, brute force on tiny inputs and
finite differences (tests/test_oracle_*.py); no function here is unpinned.
"""
from .rounding import identity, round_bf16, round_f32  # noqa: F401
