"""CPU oracle for the DAF quantize/pack path.  Test infrastructure only: nothing in the
product package may import it (tests, the smoke check and the benchmark's cpu_baseline
leg are its only callers)."""
