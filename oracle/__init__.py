"""CPU checker (test infrastructure only): plain fp64 definitions of the fused
operators, used by the tests, the smoke check and the benchmark's CPU-baseline
leg.  The GPU library does not import this package."""
