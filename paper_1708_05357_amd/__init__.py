"""DuHL hot path for MI355X: C-ABI HIP library + thin ctypes binding.

``synth`` (input generators) imports nothing from the binding; ``duhl`` loads the
HIP library on first use and fails loudly when it has not been built.
"""
__all__ = ["synth", "duhl"]
