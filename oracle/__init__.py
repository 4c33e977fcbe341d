"""CPU checker for the GPU minwise-hash library.  Test infrastructure only:
importable from tests/, the smoke check and the benchmark's CPU-baseline leg,
never from the product package."""
