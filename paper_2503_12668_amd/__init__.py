"""MI355X-native ZO2 step: thin ctypes binding over libzo2.so (HIP, gfx950).

Nothing is loaded at import; `binding.lib()` loads the shared library and fails
loudly if it has not been built (there is no CPU fallback).
"""
