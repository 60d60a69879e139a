"""CPU oracle for the basis-rotation optimizer step (TEST INFRASTRUCTURE ONLY).

Everything in this package is a plain, slow, float64 restatement of the
paper's Algorithm 1 ("Adam with basis rotation") and Algorithm 2
("Eigenbasis-Estimation").  It exists so that the HIP library can be
checked against something written independently from the paper.

Rules this package keeps:
  * it imports nothing from the product package and shares no code,
    table or helper with the HIP path;
  * only tests, the smoke entry point and the benchmark's CPU-baseline leg
    may import it -- the product never routes through it;
  * library primitives used as single steps: numpy matmul, numpy sqrt.
    The QR factorisation, the bf16 rounding and the Jacobi eigen-solver
    are written out here.
"""
