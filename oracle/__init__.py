"""CPU oracle for the RBGP4 sparse x dense product.  TEST INFRASTRUCTURE ONLY.

Nothing in the product package imports this directory; only tests/, the
smoke check and the cpu_baseline leg of bench.py may use it.
"""
