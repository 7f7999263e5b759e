"""CPU oracle of the Round Attention hot path: TEST INFRASTRUCTURE ONLY.

Nothing under this package is part of the product.  It may be imported by `tests/`, by the
smoke check and by the benchmark's CPU-baseline leg, and by nothing else; the HIP library and
its Python binding neither import it nor share any code, table or helper with it.
"""
