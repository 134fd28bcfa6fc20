"""MI355X-native decode linears over int4 group-quantised weights with a
per-layer W4A8 / W4A16 precision map.  The compute lives in libnvq.so
(hand-written HIP for gfx950, C ABI declared in include/nvq.h); this package
is the thin ctypes binding plus the seeded synthetic-input generators."""

__all__ = ["nvq", "synth"]
