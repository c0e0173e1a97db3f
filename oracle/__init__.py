"""CPU oracle (test infrastructure only): see reference.py.  Only tests, the smoke check and the
benchmark's cpu_baseline leg may import this package; the product never does."""
