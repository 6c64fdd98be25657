"""CPU oracle for C = A*B (test infrastructure only; never imported by the product)."""
