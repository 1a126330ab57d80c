"""CPU oracle for the Paillier operator path: test infrastructure only.

Nothing under this package is part of the product. Only tests, the smoke check
and the CPU-baseline leg of the benchmark may import it; the HIP library and
its Python binding never do, and the two share no code.
"""
