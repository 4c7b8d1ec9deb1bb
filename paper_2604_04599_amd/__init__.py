"""lpg: layout-propagating GEMM chains for MI355X (gfx950).

A thin Python binding over the C-ABI library built from csrc/.  The HIP library
is loaded on first use (see `api`), so importing `paper_2604_04599_amd.inputs`
alone never touches it.
"""
__all__ = ["api", "inputs", "chains"]
