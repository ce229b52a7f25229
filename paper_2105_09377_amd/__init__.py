"""MI355X-native evaluation of Glenside access-pattern programs (hand-written HIP, C ABI).

The compute lives in `csrc/` behind the C entry points declared in
`include/glenside.h`; `binding` marshals torch tensors to them.  Nothing is
imported eagerly here so that `synth` (seeded inputs) is usable without the
built library.
"""

__all__ = ["binding", "synth"]
