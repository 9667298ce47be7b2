"""CPU oracle: test infrastructure only (tests, smoke check, cpu_baseline leg).

The product package never imports this directory.
"""
