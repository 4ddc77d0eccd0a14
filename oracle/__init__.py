"""CPU oracle for the zkDL tensor-sumcheck prover (test infrastructure).

This package is the slow, obviously-correct statement of what the prover
computes, written from the paper (zkDL, arXiv 2307.16273) in Python integers
modulo the BLS12-381 scalar-field prime.  It exists to check the HIP library:
only the tests, the smoke check and the benchmark's `cpu_baseline` leg import
it.  It shares no code, constants or tables with the HIP path, and nothing in
the product imports it.

Pinned by the `-m "not gpu"` tests against: brute-force hypercube sums, the
product formula of the equality polynomial, Boolean-point evaluations, plain
integer matmul / Hadamard products, plain integer ReLU with round-half-up
rescaling, the verifier of each protocol, and NIST SHA-256 vectors.

Parity unpinned: the numeric values of Fiat-Shamir challenges.  The paper is an
interactive protocol and prints no worked numeric example, so the challenge
bytes are fixed only by the transcript format that both sides implement.
"""
