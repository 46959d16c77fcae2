"""Lookahead-decoding verification step on MI355X (gfx950), hand-written HIP behind a C ABI.

  csrc/       HIP kernels and the extern "C" entry points declared in include/la.h
  build.py    in-tree hipcc build of liblookahead.so
  binding.py  ctypes binding with the C names (argument marshalling only)
  engine.py   host-side orchestration of the calls: prefill, decode loops

Nothing here falls back to a CPU or PyTorch implementation: importing `binding` raises
if the library has not been built.
"""
