"""MI355X-native (gfx950) PruneTrain conv-layer hot path: C-ABI HIP library + thin binding.

`workloads` (synthetic input tables) imports nothing heavy; the HIP library is loaded on the
first call into `binding` and its absence is an error, never a fallback.
"""
__all__ = ["workloads", "binding"]
