"""ELSA exact linear-scan attention for MI355X (gfx950).

``paper_2604_23798_amd.elsa``   -- ctypes binding of the C-ABI HIP library (needs the built library).
``paper_2604_23798_amd.inputs`` -- seeded synthetic workloads (numpy only, no attention arithmetic).
"""
__all__ = ["inputs", "elsa"]
