"""MI355X-native HPD masked decode attention (C-ABI library + thin binding).

Importing the package loads nothing heavy; ``paper_2604_26209_amd.binding``
loads the HIP library and fails loudly when it has not been built.
"""
