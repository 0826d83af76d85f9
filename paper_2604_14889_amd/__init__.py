"""MI355X-native MemoSight decode hot path: thin Python binding over the C-ABI HIP library.

Nothing is imported eagerly; `from paper_2604_14889_amd import binding` loads the shared library.
"""
