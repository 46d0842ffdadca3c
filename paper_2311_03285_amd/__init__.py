"""Heterogeneous batched LoRA over a unified paged pool on MI355X (gfx950).

`paper_2311_03285_amd.synth` draws seeded synthetic inputs; `paper_2311_03285_amd.slora`
is the ctypes binding of the HIP library (loaded on first use, never at package import).
"""
