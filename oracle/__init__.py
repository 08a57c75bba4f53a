"""Plain, slow, fp64 CPU oracle for one sensitive-sparse zeroth-order step.

This package is TEST INFRASTRUCTURE.  It exists only so that the tests, the
smoke check and the benchmark's `cpu_baseline` leg have something obviously
correct to compare the HIP path against.  Nothing in the product package may
import it, and it imports nothing from the product package: the two share no
code, no tables and no helpers.  Inputs (activations, dense weights, targets)
are handed in as arrays by the caller.

What is computed, and where the paper defines it:

* SPSA estimator with a masked Gaussian perturbation (Definition 1,
  Definition 4) and the ZO-SGD update restricted to the fixed sensitive
  coordinates (Section 3.4, the fixed-parameter update rule).
* The linear layer in its "add the sparse part into the dequantized dense
  weight, then one dense product" form (Appendix C.5, last equation of the
  quantized group), plus the algebraically equal "dense product, then add
  the sparse product" form used as a cross-check.
* The counter-based Gaussian (Philox-4x32-10 + Box-Muller) that plays the
  role of the random-seed trick of Section 3.5.
* Two 4-bit formats for the frozen dense part (Section 3.5 allows any
  quantiser; Appendix C.5 separates uniform from non-uniform ones): uniform
  codes with group scales, and a per-row table of 16 centroids.

Pins (see tests/test_oracle_*.py): Philox known-answer vectors; both synthetic masks recomputed draw by
draw with the scalar generator; Gaussian
moments and the two SPSA moment identities of Section 3.1 / Appendix
(E g^2 = |m.c|^2 and E |g z|^2 = (k+2)|m.c|^2 for a linear loss); k = 0
reduces to a textbook dequantise-then-matmul; brute-force triple loop;
eps = 0 gives g = 0; linear loss gives g = c.z in closed form; +eps, -2eps,
+eps restores the sparse values; brute-force dense SPSA on tiny shapes;
g converges to z.grad(L) as eps -> 0.  Table format: rows with 16 levels are
reproduced bit for bit; brute-force nearest centroid with the tie rule; the
quantisation map is monotone; bins carry equal mass; the three forward forms
agree and the sparse part is added on top of the dense code.

Parity unpinned: the 10-step trajectory of the tiny configuration has no
printed worked example in the paper; it is pinned GPU-vs-oracle only.
"""
