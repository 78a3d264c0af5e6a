"""MI355X-native Stream pruning + block-sparse attention (hand-written HIP, C ABI).

Importing the package loads nothing; `paper_2510_19875_amd.binding` loads the HIP
library on first use and fails loudly when it has not been built.
"""
