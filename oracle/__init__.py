"""Reference checker for nested gradient coding (NGC) -- TEST INFRASTRUCTURE ONLY.

A plain, slow, fp64 NumPy statement of what the coded-gradient path computes,
written from the paper (Secs. II-B, II-C, III; Defs. 1-2; Alg. 1; Lemma 2) so
that a reader can check it by eye.  Nothing here is tuned, blocked or fused.

It exists to check the GPU library and to be timed beside it.  Only the test
suite, the smoke check and the benchmark's CPU-baseline leg may import it; the
GPU library never does, and the two share no code.

Pins (tests/test_oracle_*.py): closed-form and finite-difference gradients,
Def. 1 by brute force over every straggler set on small n, nesting (Def. 2),
B_0 = I, fractional-repetition worked cases, decode == sum of partial
gradients for every enumerated straggler set, layer independence.

parity unpinned: the numerical values of the random coefficients of a cyclic
B_sigma beyond the properties of Def. 1 (the paper delegates them to a cited
routine and prints no example); B is therefore handed to the library as an
input.
"""
from . import codes, coding, gradients, latency, workers  # noqa: F401
