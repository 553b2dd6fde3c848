"""Triangle Block SYRK and Large Block Cholesky for MI355X (gfx950).

`paper_2202_10217_amd.binding` marshals arguments for the C-ABI library built from
`csrc/`; `paper_2202_10217_amd.inputs` holds the seeded input generators.  Nothing
is loaded at import time: the HIP library is opened on the first call and the call
fails loudly when it has not been built.
"""
__all__ = ["binding", "inputs", "build"]
