"""CPU checker for the KV offloading hot path -- TEST INFRASTRUCTURE.

Imported only by tests, the smoke check and the benchmark's CPU-baseline leg.
"""
