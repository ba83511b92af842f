"""CPU oracle for the L-GreCo profile / solve / compress path.

TEST INFRASTRUCTURE ONLY.  Plain, slow, obviously-correct numpy code written from the
paper's statement of the method; it shares no code with the HIP path and must never be
imported by the product package.  Only tests, the smoke check and the benchmark's
cpu_baseline leg may use it.

Pinning status (what each part is checked against, other than itself):
  solver      - brute-force enumeration of every assignment, tie-break tuple included.
  quant       - closed-form per-element bound range^2/(4(2^b-1)^2), two-valued and
                constant buckets, unbiasedness / variance of stochastic rounding,
                payload round trip.  The quantizer definition itself is a reading
                (the paper names QSGD-style bucketed quantization but prints no formula).
  philox      - the known-answer vectors published with the Philox4x32-10 generator.
  topk        - brute force on tiny inputs with ties, density 1 -> zero error, energy
                conservation, paper's uniform compression ratios ~ 1/(2 d).
  lowrank     - Eckart-Young lower bound from an SVD, exact recovery of rank-rho inputs,
                full-rank -> zero error, projection identity, orthonormality.
"""
