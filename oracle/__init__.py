"""CPU oracle for the per-group-quantized linear layer (test infrastructure only).

Plain numpy, fp64 (binary32 steps emulated where the quantizer contract pins them).
Only tests, the smoke check and the benchmark's cpu_baseline leg may import this package;
it shares no code with the GPU library and imports nothing from it.

Parity pins: every function here is pinned by tests/test_oracle_*.py against published
format tables, library casts, closed forms, hand-worked examples and brute force on tiny
inputs.  No layer-level value is printed in the paper, so beyond those pins the end result
(a whole quantized layer) is "parity unpinned" against the authors' implementation.
"""
