"""MI355X-native CER / CSER matrix product (hand-written HIP kernels behind a C-ABI library).

Importing the package loads nothing; `paper_1805_10692_amd.binding` loads the built HIP library
and fails loudly when it is missing.  `paper_1805_10692_amd.workloads` only generates inputs.
"""
