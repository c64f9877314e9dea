"""MI355X-native tiered decode attention (TTKV hot path): C-ABI library + thin binding.

Nothing is loaded at import time; `binding.lib()` loads libttkv.so on first use
and raises if it has not been built."""
__all__ = ["binding", "cache", "synth", "build"]
