"""Decode-time MoE layer step with speculative expert prefetch for AMD MI355X (gfx950).

`moe_spec` is the thin ctypes binding over the C-ABI library built from `csrc/`;
`workload` holds the seeded synthetic input generators.
"""
