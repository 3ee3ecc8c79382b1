"""CPU oracle of the QoQ W4A8 hot path: test infrastructure only.

Only tests, the smoke check and the benchmark's cpu_baseline leg import this package.
It shares no code with the HIP path and the product package never imports it.
"""
