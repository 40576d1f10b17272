"""MI355X-native compressed linear layer (activation-gradient co-compression, paper Sec. 4).

Sub-modules:
  binding  thin ctypes binding over the C-ABI library (argument marshalling only)
  inputs   seeded synthetic workload generators (no method arithmetic)
  build    hipcc driver that compiles csrc/ into libacc.so

Nothing is imported eagerly: `inputs` must stay usable on machines without the
built library, and `binding` must fail loudly when the library is missing.
"""
__all__ = ["binding", "inputs", "build"]
