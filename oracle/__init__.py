"""CPU oracle for chunked-prefill attention over a paged KV cache.

Test infrastructure only: imported by tests/, by the smoke check and by the benchmark's
cpu_baseline leg.  The product package never imports this package, and this package never
imports the product.
"""
