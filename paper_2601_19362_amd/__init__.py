"""MI355X-native ODC hot path: per-layer gather and scatter-accumulate (gfx950 HIP kernels
behind a C-ABI library).  Importing the package loads nothing; `paper_2601_19362_amd.binding`
loads the built library on first use and fails loudly if it is missing."""

__all__ = ["binding", "inputs"]
