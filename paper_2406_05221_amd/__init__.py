"""Batched GCAPS / round-robin response-time analysis on MI355X (gfx950).

``binding`` wraps the C ABI of ``libgcaps_rta.so`` (hand-written HIP kernels);
``taskgen`` produces seeded synthetic tasksets; ``build`` compiles both.
"""
