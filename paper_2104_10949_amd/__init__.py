"""Replicated-share linear layers over Z_{2^64} on MI355X (gfx950).

The product is the C-ABI library declared in include/cg.h; `binding` is its thin
Python front end.  `workloads` holds the seeded synthetic inputs.
"""
