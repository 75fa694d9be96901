"""Fused deep-learning tensor operators for AMD MI355X (gfx950).

`paper_2506_10401_amd.hpct` binds the C-ABI library (HIP kernels);
`paper_2506_10401_amd.datagen` is the seeded synthetic-input generator.
Nothing is imported eagerly so the generator can be used without the library.
"""
__all__ = ["hpct", "datagen"]
