"""CPU oracle for the GEMM hot path.  Test infrastructure only: nothing in the
product package imports this, and this imports nothing from the product package."""
