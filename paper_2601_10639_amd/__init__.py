"""STEM token-indexed FFN hot path for MI355X (gfx950): C-ABI library `libstem`
plus a thin ctypes binding.  `inputs` holds the seeded synthetic workloads."""
