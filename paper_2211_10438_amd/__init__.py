"""SmoothQuant W8A8 hot path for AMD MI355X (gfx950): C-ABI HIP library + thin Python binding.

``synth`` (seeded inputs, NumPy only) imports without the native library; everything in
``binding`` needs ``libsqmi.so`` and raises loudly if it is missing.
"""
__all__ = ["synth", "binding"]
