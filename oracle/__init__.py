"""CPU oracle of the fused-operator inference path and of the placement search.

TEST INFRASTRUCTURE ONLY: the parity anchor the GPU library is checked
against.  Only the tests, the smoke check and the benchmark's cpu_baseline leg
may import it; it shares no code with the GPU path.
"""
