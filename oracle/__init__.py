"""TEST INFRASTRUCTURE ONLY: the sequential CPU oracle and its Python wrapper.

Nothing on the product path may import this package.  Only tests, the smoke check and the benchmark's
CPU-baseline leg use it.
"""
