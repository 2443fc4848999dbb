"""CPU oracle for the mixed-precision KV cache (test infrastructure only).

Nothing on the product path may import this package: it is for `tests/`, the smoke check
and the `cpu_baseline` leg of the benchmark.
"""
