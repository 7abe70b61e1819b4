"""MixKV prefill-time KV-cache compression for MI355X (gfx950).

The compute lives in `csrc/` (hand-written HIP behind a C-ABI shared library,
declared in `include/mixkv.h`); `binding` marshals arguments to it.  Nothing is
loaded at import time: `binding.lib()` loads the shared library on first use
and raises if it has not been built.
"""
__all__ = ["binding", "synth"]
