"""Packed variable-length causal attention for MI355X (gfx950).

`binding` holds the thin ctypes layer over the C-ABI library built from
`csrc/`; `workloads` holds the seeded synthetic input generators.
"""
