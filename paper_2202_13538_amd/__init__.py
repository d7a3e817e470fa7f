"""MI355X-native walk -> RPE -> join hot path of the SUREL subgraph pipeline.

The compute lives in ``csrc/`` (HIP kernels behind the C ABI declared in
``include/surel.h``); ``binding`` marshals arguments to it and ``synth`` makes
seeded synthetic inputs.  Nothing here falls back to a CPU implementation: if
the shared library is not built, loading it raises.
"""
