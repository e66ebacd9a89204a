"""Batched evaluation of candidate retention-interval assignments
(Moccasin, arXiv 2304.14463, Section 2.1) on MI355X.

`paper_2304_14463_amd.moccasin` is the binding of the C-ABI HIP library;
`paper_2304_14463_amd.inputs` generates seeded synthetic workloads.
Nothing is loaded at import time.
"""
