"""CPU oracle of the Bounded-Cache Transformer decode path (test infrastructure only).

Only tests/, the smoke check and the cpu_baseline leg of bench.py may import this package.
"""
