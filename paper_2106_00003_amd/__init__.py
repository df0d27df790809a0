"""Round-robin Givens orthogonal transforms on MI355X (gfx950).

The compute path is the HIP library built from csrc/ and declared in include/givens_rr.h;
`paper_2106_00003_amd.binding` marshals arguments to it.  Importing this package loads
nothing native; the library is loaded on first use and a missing library is an error.
"""
__all__ = ["inputs", "binding"]
